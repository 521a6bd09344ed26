"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/glowq.h declares, and rejects bad arguments with the
documented status codes before touching any device."""
import ctypes
import os
import re

import pytest

import paper_2603_25385_amd as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "glowq.h")).read() + \
        open(os.path.join(ROOT, "include", "glowq_probe.h")).read()
    declared = set(re.findall(r"\b(glowq_[a-z_0-9]+)\s*\(", text))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2603_25385_amd", "lib", "libglowq.so"))
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(G.EXPORTED)


def _unit(**kw):
    base = dict(X=0x1000, B=0x2000, T=4, d_in=256, r=16, group_size=64, act=G.GLOWQ_F16,
                out=G.GLOWQ_F32, d_out=64, ldy=64, wp=0x3000, A=0x4000, Y=0x5000, n=1)
    base.update(kw)
    mods = [G.make_module(base["wp"], base["A"], base["Y"], base["d_out"], base["ldy"])
            for _ in range(base["n"])]
    return G.make_unit(base["X"], base["B"], mods, base["T"], base["d_in"], base["r"],
                       base["group_size"], base["act"], base["out"])


def test_valid_unit_passes():
    assert G.glowq_validate_unit(_unit()) == G.GLOWQ_OK
    assert G.glowq_validate_unit(_unit(r=0, B=0, A=0)) == G.GLOWQ_OK


@pytest.mark.parametrize("kw,status", [
    (dict(X=0), G.GLOWQ_ERR_NULL), (dict(B=0), G.GLOWQ_ERR_NULL), (dict(A=0), G.GLOWQ_ERR_NULL),
    (dict(wp=0), G.GLOWQ_ERR_NULL), (dict(Y=0), G.GLOWQ_ERR_NULL),
    (dict(X=0x1008), G.GLOWQ_ERR_ALIGN), (dict(Y=0x5004), G.GLOWQ_ERR_ALIGN),
    (dict(T=0), G.GLOWQ_ERR_SHAPE), (dict(d_in=200), G.GLOWQ_ERR_SHAPE),
    (dict(group_size=32), G.GLOWQ_ERR_SHAPE), (dict(r=-8), G.GLOWQ_ERR_SHAPE),
    (dict(d_out=0), G.GLOWQ_ERR_SHAPE), (dict(ldy=56), G.GLOWQ_ERR_SHAPE),
    (dict(n=0), G.GLOWQ_ERR_SHAPE), (dict(n=9), G.GLOWQ_ERR_SHAPE),
    # well formed, but outside what the tile layout of this build holds
    (dict(d_in=192), G.GLOWQ_ERR_UNSUPPORTED), (dict(d_in=320, group_size=64), G.GLOWQ_ERR_UNSUPPORTED),
    (dict(r=12), G.GLOWQ_ERR_UNSUPPORTED), (dict(r=136), G.GLOWQ_ERR_UNSUPPORTED),
    (dict(d_out=60), G.GLOWQ_ERR_UNSUPPORTED), (dict(ldy=68), G.GLOWQ_ERR_UNSUPPORTED),
    (dict(act=G.GLOWQ_F32), G.GLOWQ_ERR_DTYPE), (dict(act=G.GLOWQ_F16, out=G.GLOWQ_BF16), G.GLOWQ_ERR_DTYPE),
])
def test_bad_units_are_rejected(kw, status):
    assert G.glowq_validate_unit(_unit(**kw)) == status
    # the forward entry points apply the same check and enqueue nothing
    with pytest.raises(G.GlowqError) as e:
        G.glowq_group_forward(_unit(**kw), True, 0x9000, 1 << 20, 0)
    assert e.value.status == status


def test_workspace_and_misc_errors():
    u = _unit()
    need = G.glowq_workspace_bytes([u])
    assert need > 0 and need % 256 == 0
    with pytest.raises(G.GlowqError) as e:
        G.glowq_group_forward(u, True, 0, 0, 0)
    assert e.value.status == G.GLOWQ_ERR_WORKSPACE
    with pytest.raises(G.GlowqError) as e:
        G.glowq_group_forward(u, True, 0x9000, need - 1, 0)
    assert e.value.status == G.GLOWQ_ERR_WORKSPACE
    with pytest.raises(G.GlowqError) as e:
        G.glowq_shared_proj(_unit(r=0, B=0, A=0), 0x8000, 0x9000, 1 << 20, 0)
    assert e.value.status == G.GLOWQ_ERR_SHAPE
    with pytest.raises(G.GlowqError) as e:
        G.glowq_prepare_weights(0, 0x10, 0x20, 64, 256, 64, 0x30, 0)
    assert e.value.status == G.GLOWQ_ERR_NULL
    with pytest.raises(G.GlowqError) as e:
        G.glowq_prepared_bytes(64, 250, 64)
    assert e.value.status == G.GLOWQ_ERR_SHAPE
    with pytest.raises(G.GlowqError) as e:
        G.glowq_prepared_bytes(64, 192, 64)
    assert e.value.status == G.GLOWQ_ERR_UNSUPPORTED
    assert G.glowq_prepared_bytes(40, 128, 128) == 3 * 1 * 272 * 4
    assert "NULL" in G.glowq_status_string(G.GLOWQ_ERR_NULL)


def test_unit_that_is_not_restored_needs_no_factors():
    """A masked unit reads neither B nor any A_i, so they may be NULL; with no restored
    unit in the call the workspace may be NULL as well.  (Checked on the host through a
    deliberately failing later argument: the call must get PAST the factor checks.)"""
    u = _unit(B=0, A=0)
    assert G.glowq_validate_unit(u) == G.GLOWQ_ERR_NULL          # as a restored unit
    bad = _unit(B=0, A=0, Y=0x5004)                              # misaligned Y comes later
    with pytest.raises(G.GlowqError) as e:
        G.glowq_group_forward(bad, False, 0, 0, 0)
    assert e.value.status == G.GLOWQ_ERR_ALIGN
    with pytest.raises(G.GlowqError) as e:
        G.glowq_group_forward(u, True, 0x9000, 1 << 20, 0)
    assert e.value.status == G.GLOWQ_ERR_NULL


def test_workspace_status_argument_checks():
    u = _unit()
    need = G.glowq_workspace_bytes([u])
    for args, status in [((0x9000, need, 0), G.GLOWQ_ERR_NULL), ((0, need, 0x8000), G.GLOWQ_ERR_NULL),
                         ((0x9000, need, 0x8002), G.GLOWQ_ERR_ALIGN),
                         ((0x9000, need - 1, 0x8000), G.GLOWQ_ERR_WORKSPACE)]:
        with pytest.raises(G.GlowqError) as e:
            G.glowq_workspace_status([u], *args)
        assert e.value.status == status


def test_workspace_holds_the_partial_results_of_k_slices():
    """A long contraction on few tiles is multiplied in slices of K (glowq.h, workspace): the
    unit's workspace then holds an fp32 slab [T][d_out] per slice and module; the rule reads
    the shapes only, and a forward call with less than that is refused before any launch."""
    plain = G.glowq_workspace_bytes([_unit(T=512, d_in=4096, d_out=4096, ldy=4096, group_size=128)])
    for d_in, slices in [(8192, 2), (11008, 2), (14336, 3), (16384, 4), (32768, 4)]:
        cut = G.glowq_workspace_bytes([_unit(T=512, d_in=d_in, d_out=4096, ldy=4096, group_size=128)])
        assert cut - plain >= slices * 512 * 4096 * 4 and cut - plain < (slices + 1) * 512 * 4096 * 4
    # not cut: few tokens, a short contraction, more than 128 tiles
    for kw in [dict(T=64, d_in=14336, d_out=4096, ldy=4096), dict(T=512, d_in=8064, d_out=4096, ldy=4096),
               dict(T=1024, d_in=14336, d_out=5120, ldy=5120)]:
        assert G.glowq_workspace_bytes([_unit(group_size=128, **kw)]) < plain * 3
    u = _unit(T=512, d_in=14336, d_out=4096, ldy=4096, group_size=128)
    with pytest.raises(G.GlowqError) as e:
        G.glowq_group_forward(u, True, 0x10000, plain, 0)
    assert e.value.status == G.GLOWQ_ERR_WORKSPACE


def test_layerwise_argument_checks():
    """The layer-wise mode forwards the unit's modules as one-module units: its workspace
    is the sum of theirs, and every module needs a right factor of its own."""
    u = _unit(n=3)
    solo = G.glowq_workspace_bytes([_unit(n=1)])
    need = G.glowq_layerwise_workspace_bytes([u, u])
    assert need == 6 * solo
    with pytest.raises(G.GlowqError) as e:                       # a rank-0 unit has nothing to compare
        G.glowq_layerwise_workspace_bytes([u, _unit(r=0, B=0, A=0)])
    assert e.value.status == G.GLOWQ_ERR_SHAPE
    ok = [0x2000, 0x2100, 0x2200, 0x2300, 0x2400, 0x2500]
    cases = [((ok[:4] + [0] + ok[5:], 0x9000, need), G.GLOWQ_ERR_NULL),
             ((ok[:5] + [0x2504], 0x9000, need), G.GLOWQ_ERR_ALIGN),
             ((ok, 0x9000, need - 16), G.GLOWQ_ERR_WORKSPACE),
             ((ok, 0, need), G.GLOWQ_ERR_WORKSPACE)]
    for args, status in cases:
        with pytest.raises(G.GlowqError) as e:
            G.glowq_layerwise_forward([u, u], *args, 0)
        assert e.value.status == status, args
    with pytest.raises(G.GlowqError) as e:                       # unsupported shapes stay unsupported
        G.glowq_layerwise_forward([_unit(n=2, d_in=192)], [0x2000, 0x2100], 0x9000, 1 << 20, 0)
    assert e.value.status == G.GLOWQ_ERR_UNSUPPORTED


def test_select_units_is_the_oracles_selection():
    from oracle import glowq_oracle as O
    import numpy as np
    rng = np.random.default_rng(3)
    for n in (1, 2, 7, 40):
        s = np.round(rng.random(n), 1)                # many ties
        for k in (0, 1, n // 2, n, n + 3):
            assert G.glowq_select_units(s.tolist(), k) == O.select_units(s, k).tolist()
    with pytest.raises(G.GlowqError) as e:
        G.glowq_select_units([0.5], -1)
    assert e.value.status == G.GLOWQ_ERR_SHAPE


def test_unit_importance_argument_checks():
    u = _unit(n=2)
    for args, status in [(([0x7000, 0], 0x9000, 0xA000), G.GLOWQ_ERR_NULL),
                         (([0x7000, 0x7100], 0, 0xA000), G.GLOWQ_ERR_NULL),
                         (([0x7000, 0x7100], 0x9004, 0xA000), G.GLOWQ_ERR_ALIGN),
                         (([0x7000, 0x7104], 0x9000, 0xA000), G.GLOWQ_ERR_ALIGN)]:
        with pytest.raises(G.GlowqError) as e:
            G.glowq_unit_importance(u, *args, 0)
        assert e.value.status == status, args
    with pytest.raises(G.GlowqError) as e:
        G.glowq_unit_importance(_unit(B=0), [0x7000], 0x9000, 0xA000, 0)
    assert e.value.status == G.GLOWQ_ERR_NULL


def test_quantize_rtn_argument_checks():
    ok = (0x7000, 64, 256, 128, 0x8000, 0x9000, 0xA000)
    for i, status in [(0, G.GLOWQ_ERR_NULL), (4, G.GLOWQ_ERR_NULL), (5, G.GLOWQ_ERR_NULL), (6, G.GLOWQ_ERR_NULL)]:
        a = list(ok)
        a[i] = 0
        with pytest.raises(G.GlowqError) as e:
            G.glowq_quantize_rtn(*a)
        assert e.value.status == status
    for a, status in [((0x7004,) + ok[1:], G.GLOWQ_ERR_ALIGN),
                      (ok[:3] + (32,) + ok[4:], G.GLOWQ_ERR_SHAPE),
                      (ok[:2] + (200,) + ok[3:], G.GLOWQ_ERR_SHAPE),
                      (ok[:1] + (0,) + ok[2:], G.GLOWQ_ERR_SHAPE),
                      (ok[:2] + (192, 64) + ok[4:], G.GLOWQ_ERR_UNSUPPORTED),
                      (ok[:1] + (60,) + ok[2:], G.GLOWQ_ERR_UNSUPPORTED)]:
        with pytest.raises(G.GlowqError) as e:
            G.glowq_quantize_rtn(*a)
        assert e.value.status == status, a


def test_factorize_argument_checks():
    u = _unit(n=2, d_out=64, d_in=256)                       # m = 128 rows, d = 256
    nbytes = G.glowq_factorize_workspace_bytes(u, 16, 8)
    assert nbytes > 128 * 256 * 8 and nbytes % 256 == 0      # holds at least the float64 stack
    assert G.glowq_factorize_workspace_bytes(u, 16, 24) > nbytes
    good = dict(W=[0x7000, 0x7100], sx=0, r=16, p=8, q=2, Om=0xB000, ws=0xC000, nb=nbytes,
                A=[0xD000, 0xD100], B=0xE000, sig=0xF000)

    def call(**kw):
        a = dict(good)
        a.update(kw)
        G.glowq_factorize_unit(u, a["W"], a["sx"], a["r"], a["p"], a["q"], a["Om"], a["ws"], a["nb"],
                               a["A"], a["B"], a["sig"], 0)

    for kw, status in [(dict(Om=0), G.GLOWQ_ERR_NULL), (dict(B=0), G.GLOWQ_ERR_NULL),
                       (dict(W=[0x7000, 0]), G.GLOWQ_ERR_NULL), (dict(A=[0, 0xD100]), G.GLOWQ_ERR_NULL),
                       (dict(ws=0), G.GLOWQ_ERR_WORKSPACE), (dict(nb=nbytes - 1), G.GLOWQ_ERR_WORKSPACE),
                       (dict(ws=0xC010), G.GLOWQ_ERR_ALIGN), (dict(Om=0xB004), G.GLOWQ_ERR_ALIGN),
                       (dict(sx=0xB104), G.GLOWQ_ERR_ALIGN), (dict(W=[0x7000, 0x7108]), G.GLOWQ_ERR_ALIGN),
                       (dict(r=0), G.GLOWQ_ERR_SHAPE), (dict(p=-1), G.GLOWQ_ERR_SHAPE),
                       (dict(q=-1), G.GLOWQ_ERR_SHAPE),
                       (dict(r=136, p=0), G.GLOWQ_ERR_SHAPE),          # more ranks than the stack has rows
                       (dict(r=128, p=200), G.GLOWQ_ERR_SHAPE),        # sketch wider than d_in
                       (dict(r=12), G.GLOWQ_ERR_UNSUPPORTED), (dict(q=9), G.GLOWQ_ERR_UNSUPPORTED)]:
        with pytest.raises(G.GlowqError) as e:
            call(**kw)
        assert e.value.status == status, kw
    wide = _unit(n=4, d_out=512, ldy=512, d_in=1024)
    with pytest.raises(G.GlowqError) as e:
        G.glowq_factorize_workspace_bytes(wide, 128, 136)   # r + p above the sketch limit
    assert e.value.status == G.GLOWQ_ERR_UNSUPPORTED


def test_mx_argument_checks():
    assert G.glowq_mx_prepared_bytes(64, 256) == 4 * 2 * (1024 + 64)        # 4 row blocks x 2 tiles
    assert G.glowq_mx_prepared_bytes(40, 256) == 3 * 2 * (1024 + 64)        # a ragged last row block
    for a, status in [((64, 200), G.GLOWQ_ERR_SHAPE), ((0, 256), G.GLOWQ_ERR_SHAPE),
                      ((64, 160), G.GLOWQ_ERR_UNSUPPORTED), ((60, 256), G.GLOWQ_ERR_UNSUPPORTED)]:
        with pytest.raises(G.GlowqError) as e:
            G.glowq_mx_prepared_bytes(*a)
        assert e.value.status == status, a
    for a, status in [((0, 0x8000, 64, 256, 0x9000), G.GLOWQ_ERR_NULL), ((0x7000, 0, 64, 256, 0x9000), G.GLOWQ_ERR_NULL),
                      ((0x7000, 0x8000, 64, 256, 0), G.GLOWQ_ERR_NULL), ((0x7004, 0x8000, 64, 256, 0x9000), G.GLOWQ_ERR_ALIGN),
                      ((0x7000, 0x8001, 64, 256, 0x9000), None)]:
        if status is None:
            continue                                     # (scale bytes need no alignment; the call would run)
        with pytest.raises(G.GlowqError) as e:
            G.glowq_mx_prepare_weights(*a)
        assert e.value.status == status, a
    for a, status in [((0, 4, 256, G.GLOWQ_F16, 0x8000, 0x9000), G.GLOWQ_ERR_NULL),
                      ((0x7000, 0, 256, G.GLOWQ_F16, 0x8000, 0x9000), G.GLOWQ_ERR_SHAPE),
                      ((0x7000, 4, 250, G.GLOWQ_F16, 0x8000, 0x9000), G.GLOWQ_ERR_SHAPE),
                      ((0x7000, 4, 256, G.GLOWQ_F32, 0x8000, 0x9000), G.GLOWQ_ERR_DTYPE),
                      ((0x7000, 4, 256, G.GLOWQ_F16, 0x8004, 0x9000), G.GLOWQ_ERR_ALIGN)]:
        with pytest.raises(G.GlowqError) as e:
            G.glowq_mx_quantize_activations(*a)
        assert e.value.status == status, a
    u = _unit(group_size=0, T=16)                        # the group size plays no part here
    nb = G.glowq_mx_workspace_bytes(u)
    assert nb % 256 == 0 and nb >= 16 * 256 + 16 * 8
    assert G.glowq_mx_workspace_bytes(_unit(group_size=0, T=300)) > 300 * 256        # holds the quantised activations
    for kw, args, status in [(dict(), (0, nb), G.GLOWQ_ERR_WORKSPACE), (dict(), (0xC000, nb - 1), G.GLOWQ_ERR_WORKSPACE),
                             (dict(), (0xC010, nb), G.GLOWQ_ERR_ALIGN), (dict(B=0), (0xC000, nb), G.GLOWQ_ERR_NULL),
                             (dict(r=12), (0xC000, nb), G.GLOWQ_ERR_UNSUPPORTED)]:
        with pytest.raises(G.GlowqError) as e:
            G.glowq_mx_group_forward(_unit(group_size=0, **{"T": 16, **kw}), 1, *args)
        assert e.value.status == status, (kw, args)
