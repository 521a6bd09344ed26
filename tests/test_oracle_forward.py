"""Pins for the oracle's forward (Sec. 3.3, Eqs. 8-9) and for the restore gating
of GlowQ-S: special cases with a textbook answer, brute force on tiny shapes,
identities the paper states, and agreement between the two oracle forms (numpy
matmul and the naive C loops), which share no code."""
import numpy as np
import pytest

from glowq_inputs import CONFIGS, UnitShape
from oracle import glowq_oracle as O
from util import recipe_unit, rel_err


def _tiny_unit(seed=0, T=3, d=16, d_outs=(4, 12), r=2, G=8, act="f16"):
    rng = np.random.default_rng(seed)
    W = [(rng.standard_normal((o, d)) * 0.02).astype(np.float32) for o in d_outs]
    X = O.f64_to_bits(rng.standard_normal((T, d)) * np.exp(0.5 * rng.standard_normal(d)), act)
    u = O.build_unit(W, X, r, G, act)
    u["W"] = W
    return u


def _brute_force(unit, restore=True):
    """Eq. 9 expanded by hand with Python floats, summed output-major and with the
    correction folded per rank index (a different order from both oracle forms)."""
    act, G = unit["act"], unit["G"]
    X = O.bits_to_f64(unit["X"], act).tolist()
    B = O.bits_to_f64(unit["B"], act).tolist()
    T, d, r = len(X), unit["d_in"], unit["r"]
    outs = []
    for m in unit["modules"]:
        s = O.bits_to_f64(m["scales"], "f16").tolist()
        z = O.bits_to_f64(m["zeros"], "f16").tolist()
        A = O.bits_to_f64(m["A"], act).tolist()
        words = m["wq"].tolist()
        n_out = len(words)
        Y = [[0.0] * n_out for _ in range(T)]
        for o in range(n_out):
            wrow = []
            for k in range(d):
                qv = (words[o][k // 8] >> (4 * (k % 8))) & 15
                v = (qv - z[o][k // G]) * s[o][k // G]
                wrow.append(float(O.bits_to_f64(O.f64_to_bits(np.float64(v), act), act)))
            for t in range(T):
                acc = 0.0
                for k in reversed(range(d)):
                    acc += wrow[k] * X[t][k]
                if restore:
                    for j in range(r):
                        rj = 0.0
                        for k in range(d):
                            rj += B[j][k] * X[t][k]
                        acc += A[o][j] * rj
                Y[t][o] = acc
        outs.append(np.array(Y))
    return outs


@pytest.mark.parametrize("act", ["f16", "bf16"])
def test_brute_force_tiny(act, naive):
    u = _tiny_unit(act=act)
    for restore in (True, False):
        ref = _brute_force(u, restore)
        a = O.group_forward(u, restore)
        b = naive.group_forward(u, restore)
        for y_ref, ya, yb in zip(ref, a, b):
            assert ya.shape == y_ref.shape == yb.shape
            assert np.allclose(ya, y_ref, rtol=1e-13, atol=1e-15)
            assert np.allclose(yb, y_ref, rtol=1e-13, atol=1e-15)


def test_integer_special_case_is_an_exact_integer_product(naive):
    # s = 1, z = 0, r = 0, integer X: Y = X q^T exactly
    rng = np.random.default_rng(1)
    q = rng.integers(0, 16, size=(24, 64), dtype=np.uint8)
    Xi = rng.integers(-8, 9, size=(5, 64))
    unit = dict(X=O.f64_to_bits(Xi.astype(np.float64), "f16"), B=np.zeros((0, 64), np.uint16),
                act="f16", G=64, r=0, d_in=64, T=5,
                modules=[dict(wq=O.pack_int4(q), scales=O.f64_to_bits(np.ones((24, 1)), "f16"),
                              zeros=O.f64_to_bits(np.zeros((24, 1)), "f16"),
                              A=np.zeros((24, 0), np.uint16))])
    ref = Xi @ q.astype(np.int64).T
    assert np.array_equal(O.group_forward(unit)[0], ref.astype(np.float64))
    assert np.array_equal(naive.group_forward(unit)[0], ref.astype(np.float64))


def test_rank_zero_and_masked_unit_reduce_to_plain_dequantised_product(naive):
    u = _tiny_unit(seed=2, T=4, d=32, d_outs=(8, 8, 16), r=4)
    plain = [O.bits_to_f64(u["X"], "f16") @ O.dequant(O.unpack_int4(m["wq"]), m["scales"],
                                                        m["zeros"], u["G"], "f16").T
             for m in u["modules"]]
    masked = O.group_forward(u, restore=False)
    u0 = dict(u, r=0)
    rank0 = O.group_forward(u0, restore=True)
    for p, a, b, c in zip(plain, masked, rank0, naive.group_forward(u, restore=False)):
        assert np.array_equal(a, p) and np.array_equal(b, p)
        assert np.allclose(c, p, rtol=1e-13, atol=1e-16)
    # the restored output differs from the masked one by exactly R A_i^T
    full = O.group_forward(u, restore=True)
    R = O.shared_proj(u["X"], u["B"], "f16")
    for m, f, p in zip(u["modules"], full, plain):
        assert np.allclose(f - p, R @ O.bits_to_f64(m["A"], "f16").T, rtol=1e-12, atol=1e-15)
        assert np.max(np.abs(f - p)) > 0


def test_full_rank_unrounded_factors_recover_the_unquantised_product():
    # with A_i B = E_i the corrected output is W_i X (Sec. 3: W ~ W_q + A B)
    rng = np.random.default_rng(3)
    d, T = 32, 6
    W = [(rng.standard_normal((o, d)) * 0.02).astype(np.float32) for o in (24, 40)]
    Xb = O.f64_to_bits(rng.standard_normal((T, d)), "f16")
    X = O.bits_to_f64(Xb, "f16")
    What = []
    for w in W:
        q, s, z = O.quantize_rtn(w, 16)
        What.append(O.dequant(q, s, z, 16, "f16"))
    E = O.stack_errors(W, What)
    A, B, _ = O.factors_svd(E, d)
    R = X @ B.T
    for w, wh, A_i in zip(W, What, O.split_rows(A, [24, 40])):
        y = X @ wh.T + R @ A_i.T
        ref = X @ w.astype(np.float64).T
        assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref)) + 1e-14
        # and the quantised product alone is visibly off
        assert np.max(np.abs(X @ wh.T - ref)) > 1e-4


def test_rank_r_correction_removes_the_leading_error_energy():
    # stored (rounded) factors of rank r shrink ||Y - W X|| compared with no correction
    u = recipe_unit(O, 1, 0, 16)
    X = O.bits_to_f64(u["X"], "f16")
    on = O.group_forward(u, True)
    off = O.group_forward(u, False)
    for W, y1, y0 in zip(u["W"], on, off):
        ref = X @ W.astype(np.float64).T
        assert np.linalg.norm(y1 - ref) < 0.97 * np.linalg.norm(y0 - ref)


def _tiny_layerwise_unit(seed=11, T=4, d=32, d_outs=(8, 16, 8), r=4, G=16, act="f16"):
    rng = np.random.default_rng(seed)
    W = [(rng.standard_normal((o, d)) * 0.02).astype(np.float32) for o in d_outs]
    X = O.f64_to_bits(rng.standard_normal((T, d)) * np.exp(0.5 * rng.standard_normal(d)), act)
    u = O.build_unit_layerwise(W, X, r, G, act)
    u["W"] = W
    return u


@pytest.mark.parametrize("act", ["f16", "bf16"])
def test_layerwise_forward_uses_each_modules_own_factors(act):
    # brute force, module by module, with that module's B_i in the place of the shared B
    u = _tiny_layerwise_unit(act=act)
    got = O.layerwise_forward(u)
    assert len({m["B"].tobytes() for m in u["modules"]}) == len(u["modules"])
    for m, y in zip(u["modules"], got):
        solo = dict(u, B=m["B"], modules=[m])
        (ref,) = _brute_force(solo, True)
        assert y.shape == ref.shape
        assert np.allclose(y, ref, rtol=1e-13, atol=1e-15)
        # a solo unit's group forward is the same thing
        assert np.array_equal(O.group_forward(solo, True)[0], y)


def test_layerwise_factors_are_each_blocks_best_rank_r():
    # Eckart-Young per block: ||E_i - A_i B_i||_F^2 is the tail energy of E_i's spectrum,
    # and no shared right factor does better on any block (Prop. 1 bounds the stack, the
    # per-block optimum bounds each block)
    r, G, act = 4, 16, "f16"
    u = _tiny_layerwise_unit(r=r, G=G, act=act)
    shared = O.build_unit(u["W"], u["X"], r, G, act)
    Bs = O.bits_to_f64(shared["B"], act)
    for W, m, ms in zip(u["W"], u["modules"], shared["modules"]):
        What = O.dequant(O.unpack_int4(m["wq"]), m["scales"], m["zeros"], G, act)
        E = W.astype(np.float64) - What
        sv = np.linalg.svd(E, compute_uv=False)
        tail = float(np.sum(sv[r:] ** 2))
        A_i, B_i = O.bits_to_f64(m["A"], act), O.bits_to_f64(m["B"], act)
        own = float(np.linalg.norm(E - A_i @ B_i) ** 2)
        assert abs(own - tail) <= 2e-3 * float(np.sum(sv ** 2))      # 16-bit storage of the factors
        sh = float(np.linalg.norm(E - O.bits_to_f64(ms["A"], act) @ Bs) ** 2)
        assert own <= sh * (1 + 1e-3)
        # balanced split (Eq. 7): both factors carry the square roots of the singular values
        assert np.allclose(np.linalg.norm(A_i, axis=0), np.sqrt(sv[:r]), rtol=2e-3)
        assert np.allclose(np.linalg.norm(B_i, axis=1), np.sqrt(sv[:r]), rtol=2e-3)


def test_layerwise_setup_of_a_single_module_is_the_shared_setup():
    rng = np.random.default_rng(5)
    W = [(rng.standard_normal((24, 64)) * 0.02).astype(np.float32)]
    X = O.f64_to_bits(rng.standard_normal((3, 64)), "f16")
    a = O.build_unit(W, X, 8, 32, "f16")
    b = O.build_unit_layerwise(W, X, 8, 32, "f16")
    # (singular vectors are fixed up to a sign per rank; the products are unique)
    Pa = O.bits_to_f64(a["modules"][0]["A"], "f16") @ O.bits_to_f64(a["B"], "f16")
    Pb = O.bits_to_f64(b["modules"][0]["A"], "f16") @ O.bits_to_f64(b["modules"][0]["B"], "f16")
    assert np.allclose(Pa, Pb, rtol=0, atol=1e-12)
    for ya, yb in zip(O.group_forward(a), O.layerwise_forward(b)):
        assert np.allclose(ya, yb, rtol=1e-12, atol=1e-14)


def test_shared_projection_equals_per_module_projection(naive):
    u = _tiny_unit(seed=4, T=5, d=64, d_outs=(16, 8, 8), r=8, G=32)
    shared = O.group_forward(u, True)
    layerwise = O.layerwise_forward(u)
    for a, b in zip(shared, layerwise):
        assert np.array_equal(a, b)
    R = O.shared_proj(u["X"], u["B"], "f16")
    assert R.shape == (5, 8)
    assert np.allclose(R, naive.shared_proj(u["X"], u["B"], "f16"), rtol=1e-13, atol=1e-16)
    # R[t][j] is row t of X against row j of B (not the transpose): plant a probe
    Xp = np.zeros((2, 64)); Xp[1, 3] = 2.0
    Bp = np.zeros((8, 64)); Bp[5, 3] = 0.5
    Rp = O.shared_proj(O.f64_to_bits(Xp, "f16"), O.f64_to_bits(Bp, "f16"), "f16")
    expect = np.zeros((2, 8)); expect[1, 5] = 1.0
    assert np.array_equal(Rp, expect)


def test_block_forward_applies_the_mask_per_unit():
    units = [_tiny_unit(seed=s, d_outs=(8,) if s % 2 else (8, 8)) for s in range(4)]
    mask = [1, 0, 0, 1]
    out = O.block_forward(units, mask)
    for u, f, ys in zip(units, mask, out):
        ref = O.group_forward(u, bool(f))
        other = O.group_forward(u, not f)
        for y, a, b in zip(ys, ref, other):
            assert np.array_equal(y, a) and not np.array_equal(y, b)


def test_token_independence_and_reparameterisation():
    u = _tiny_unit(seed=5, T=4, d=32, d_outs=(8, 24), r=4)
    full = O.group_forward(u)
    for t in range(4):
        ut = dict(u, X=u["X"][t:t + 1], T=1)
        for y, yt in zip(full, O.group_forward(ut)):
            assert np.allclose(y[t], yt[0], rtol=1e-13, atol=1e-16)
    # (A G, G^-1 B) with orthogonal G leaves A B unchanged (Lemma A.1.4); checked on
    # unrounded factors through the definition
    rng = np.random.default_rng(6)
    Gm, _ = np.linalg.qr(rng.standard_normal((4, 4)))
    A = O.bits_to_f64(u["modules"][0]["A"], "f16")
    B = O.bits_to_f64(u["B"], "f16")
    X = O.bits_to_f64(u["X"], "f16")
    assert np.allclose((X @ B.T) @ A.T, (X @ (Gm.T @ B).T) @ (A @ Gm).T, atol=1e-14)


@pytest.mark.parametrize("cfg_id", [1])
def test_numpy_and_c_forms_agree_on_the_tiny_workload(cfg_id, naive):
    cfg = CONFIGS[cfg_id]
    u = recipe_unit(O, cfg_id, 0, cfg["T"][0])
    a = O.group_forward(u)
    b = naive.group_forward(u)
    for ya, yb in zip(a, b):
        assert rel_err(yb, ya) < 1e-12
    rows = [np.array([0, 7, 255], np.int32)] * 3
    c = naive.group_forward(u, rows=rows)
    for ya, yc in zip(a, c):
        assert np.allclose(yc, ya[:, [0, 7, 255]], rtol=1e-12, atol=1e-14)


def test_non_square_shapes_catch_transposed_operands(naive):
    shape = UnitShape("g", 64, (32, 96))
    u = recipe_unit(O, 1, 0, 5, r=8, shape=shape, G=32)
    ys = O.group_forward(u)
    assert [y.shape for y in ys] == [(5, 32), (5, 96)]
    for y, yc in zip(ys, naive.group_forward(u)):
        assert rel_err(yc, y) < 1e-12
    assert u["B"].shape == (8, 64) and u["modules"][1]["A"].shape == (96, 8)
    assert u["modules"][1]["wq"].shape == (96, 8) and u["modules"][1]["scales"].shape == (96, 2)
