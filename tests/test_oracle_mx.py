"""Pins of the microscaling oracle (MXFP4 weights, MXFP8 activations; the formats of the
OCP MX v1.0 specification that the paper's datatype appendix refers to) against things
other than itself: the specification's value tables, a library's float8 cast, brute-force
nearest-value search, a block worked by hand, and closed-form special cases."""
import os

import numpy as np
import pytest
import torch

from oracle import glowq_oracle as O
from oracle import mx_oracle as MX

HERE = os.path.dirname(os.path.abspath(__file__))


def test_e2m1_table_is_the_specifications():
    v = MX.element_values("e2m1")
    assert v[:8].tolist() == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert np.array_equal(v[8:], -v[:8]) and np.signbit(v[8])


def test_e4m3_values_against_the_library_type():
    v = MX.element_values("e4m3")
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(v), np.isnan(ref)) and int(np.isnan(v).sum()) == 2
    ok = ~np.isnan(v)
    assert np.array_equal(v[ok], ref[ok])
    assert np.nanmax(v) == 448.0 and v[1] == 2.0 ** -9          # largest finite, smallest subnormal


def test_e8m0_scale_values():
    assert MX.scale_values(np.array([0, 127, 128, 254])).tolist() == [2.0 ** -127, 1.0, 2.0, 2.0 ** 127]


def test_round_to_e4m3_against_the_library_cast():
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.standard_normal(20000) * 50, rng.standard_normal(20000) * 0.01,
                        rng.uniform(-448, 448, 20000)]).astype(np.float32)
    v = v[np.abs(v) <= 448]
    # every midpoint between neighbouring values too (ties)
    grid = np.sort(MX.element_values("e4m3")[:127])
    mids = ((grid[1:] + grid[:-1]) / 2).astype(np.float32)
    v = np.concatenate([v, mids, -mids, grid.astype(np.float32)])
    ref = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = MX.round_to_element(v.astype(np.float64), "e4m3")
    # (the library keeps the sign of a value that rounds to zero; the oracle's zero is +0)
    same = (got == ref) | ((ref & 0x7F) == 0) & (got == 0)
    assert same.all()
    # saturation instead of the library's NaN above the largest finite value
    assert MX.round_to_element(np.array([449.0, 1e6, -500.0]), "e4m3").tolist() == [0x7E, 0x7E, 0xFE]


def test_round_to_e2m1_by_brute_force():
    mags = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    v = np.concatenate([np.linspace(-7.5, 7.5, 6001), (mags[1:] + mags[:-1]) / 2, -(mags[1:] + mags[:-1]) / 2])
    got = MX.round_to_element(v, "e2m1")
    for x, c in zip(v, got):
        d = np.abs(np.abs(x) - mags)
        best = np.flatnonzero(d == d.min())
        code = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]   # tie: the even code
        if abs(x) > 6:
            code = 7
        want = code | (8 if (x < 0 and code != 0) else 0)
        assert c == want, (x, c, want)


def test_worked_block():
    txt = dict(l.split(" = ") for l in open(os.path.join(HERE, "golden", "mxfp4_worked_example.txt"))
               if " = " in l and not l.startswith("#"))
    vals = np.zeros(32)
    given = np.array([float(t) for t in txt["values"].split()])
    vals[:len(given)] = given
    codes, scales = MX.mx_quantize(vals[None, :], "e2m1")
    assert scales[0, 0] == int(txt["scale_code"])
    assert codes[0, :len(given)].tolist() == [int(t) for t in txt["codes"].split()]
    assert not codes[0, len(given):].any()


@pytest.mark.parametrize("fmt", ["e2m1", "e4m3"])
def test_quantiser_invariants(fmt):
    f = MX.FORMATS[fmt]
    rng = np.random.default_rng(1)
    V = rng.standard_normal((40, 256)) * np.exp(rng.standard_normal((40, 1)) * 3)
    V[3, 64:96] = 0.0                                            # a block of zeros
    V[4, 0:32] = 2.0 ** -140                                     # below the smallest scale
    codes, scales = MX.mx_quantize(V, fmt)
    assert scales.shape == (40, 8) and scales.max() <= 254 and scales[3, 2] == 127
    deq = MX.mx_dequant(codes, scales, fmt)
    assert not deq[3, 64:96].any()
    # the largest element of a block lands in the format's top binade (or saturates)
    vals = np.abs(MX.element_values(fmt)[codes.astype(int)]).reshape(40, 8, 32).max(axis=2)
    live = (np.abs(V).reshape(40, 8, 32).max(axis=2) > 0) & (scales > 0)
    assert np.all(vals[live] >= 2.0 ** f["emax"]) and np.all(vals[live] <= f["vmax"])
    # error: half a quantum of the element's binade, except where the value was clamped
    S = np.repeat(MX.scale_values(scales), 32, axis=1)
    a = np.abs(V) / S
    clamped = a > f["vmax"]
    e = np.maximum(np.floor(np.log2(np.where(a > 0, a, 1.0))), 1 - f["bias"])
    assert np.all(np.abs(V - deq)[~clamped] <= (S * 2.0 ** (e - f["mbits"]) / 2)[~clamped] * (1 + 1e-12))
    assert np.all(np.abs(deq)[clamped] == (f["vmax"] * S)[clamped])
    # values on the grid come back unchanged, codes and scales too
    c2, s2 = MX.mx_quantize(deq, fmt)
    assert np.array_equal(MX.mx_dequant(c2, s2, fmt), deq)


def test_forward_by_loops_and_special_cases():
    rng = np.random.default_rng(2)
    T, d, r = 3, 64, 8
    W = [rng.standard_normal((8, d)) * 0.02, rng.standard_normal((16, d)) * 0.02]
    Xb = O.f64_to_bits(rng.standard_normal((T, d)), "f16")
    u = MX.build_unit_mx(W, Xb, r, "f16")
    Y = MX.mx_group_forward(u)
    X = O.bits_to_f64(Xb, "f16")
    xc, xs = MX.mx_quantize(X, "e4m3")
    e4, e2 = MX.element_values("e4m3"), MX.element_values("e2m1")
    Bm = O.bits_to_f64(u["B"], "f16")
    for m, Ym in zip(u["modules"], Y):
        A = O.bits_to_f64(m["A"], "f16")
        for t in range(T):
            for o in range(m["d_out"]):
                acc = 0.0
                for k in range(d):
                    acc += e4[xc[t, k]] * 2.0 ** (int(xs[t, k // 32]) - 127) * e2[m["codes"][o, k]] * 2.0 ** (int(m["scales"][o, k // 32]) - 127)
                for j in range(r):
                    acc += sum(X[t, k] * Bm[j, k] for k in range(d)) * A[o, j]
                assert Ym[t, o] == pytest.approx(acc, rel=1e-12, abs=1e-15)
    # not restored: the main product alone
    Y0 = MX.mx_group_forward(u, restore=False)
    u0 = dict(u, r=0)
    assert all(np.array_equal(a, b) for a, b in zip(Y0, MX.mx_group_forward(u0)))
    # activations and weights that sit on the grids: the product of the inputs themselves
    Xg = MX.mx_dequant(*MX.mx_quantize(rng.standard_normal((T, d)), "e4m3"), "e4m3")
    Wg = MX.mx_dequant(*MX.mx_quantize(rng.standard_normal((8, d)), "e2m1"), "e2m1")
    ug = MX.build_unit_mx([Wg], O.f64_to_bits(Xg, "bf16"), 0, "bf16")     # (e4m3 values fit bf16)
    assert np.array_equal(O.bits_to_f64(ug["X"], "bf16"), Xg)
    assert np.allclose(MX.mx_group_forward(ug)[0], Xg @ Wg.T, rtol=1e-14, atol=0)
    # the stored factors reduce the weight error as Eckart-Young says
    E = O.stack_errors(W, [MX.mx_dequant(m["codes"], m["scales"], "e2m1") for m in u["modules"]])
    s = np.linalg.svd(E, compute_uv=False)
    A = np.concatenate([O.bits_to_f64(m["A"], "f16") for m in u["modules"]])
    assert np.linalg.norm(E - A @ Bm, "fro") == pytest.approx(np.sqrt(np.sum(s[r:] ** 2)), rel=5e-3)
