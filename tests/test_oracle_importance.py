"""Pins for the oracle's importance scores and the GlowQ-S selection (Sec. 3.3,
Eqs. 10-11): closed forms, invariants and brute force."""
import itertools

import numpy as np
import pytest

from oracle import glowq_oracle as O


def _unit_weights(seed=0, d=64, d_outs=(24, 8, 16), G=32):
    rng = np.random.default_rng(seed)
    W = [(rng.standard_normal((o, d)) * 0.02).astype(np.float32) for o in d_outs]
    What = []
    for w in W:
        q, s, z = O.quantize_rtn(w, G)
        What.append(O.dequant(q, s, z, G, "f16"))
    return W, What


def test_ner_is_the_ratio_of_two_plain_sums():
    W, What = _unit_weights()
    e = w = 0.0
    for a, b in zip(W, What):                       # element by element, Python floats
        for x, y in zip(a.astype(np.float64).ravel().tolist(), b.ravel().tolist()):
            e += (x - y) * (x - y)
            w += x * x
    assert O.importance_ner(W, What) == pytest.approx(e / w, rel=1e-12)


def test_ner_special_cases():
    rng = np.random.default_rng(1)
    W = [rng.standard_normal((8, 16))]
    assert O.importance_ner(W, W) == 0.0                        # nothing lost
    assert O.importance_ner(W, [np.zeros((8, 16))]) == pytest.approx(1.0, rel=1e-15)   # everything lost
    assert O.importance_ner(W, [2 * W[0]]) == pytest.approx(1.0, rel=1e-15)            # E = -W
    # scale invariance and the stacking of modules: a module pair is one unit
    W2 = [rng.standard_normal((4, 16)), rng.standard_normal((6, 16))]
    Wh2 = [w + 0.01 * rng.standard_normal(w.shape) for w in W2]
    g = O.importance_ner(W2, Wh2)
    assert O.importance_ner([3 * w for w in W2], [3 * w for w in Wh2]) == pytest.approx(g, rel=1e-12)
    stacked = O.importance_ner([np.concatenate(W2)], [np.concatenate(Wh2)])
    assert stacked == pytest.approx(g, rel=1e-12)


def test_ner_of_uniform_rounding_noise():
    # a uniform quantiser of step s leaves an error of variance s^2 / 12
    rng = np.random.default_rng(2)
    W = rng.uniform(-1, 1, size=(256, 256))
    step = 1.0 / 64
    What = np.round(W / step) * step
    expected = (step ** 2 / 12) / (1.0 / 3)                     # var of U(-1, 1) is 1/3
    assert O.importance_ner([W], [What]) == pytest.approx(expected, rel=0.03)


@pytest.mark.parametrize("seed", [0, 3])
def test_ec_bounds_monotonicity_and_saturation(seed):
    W, What = _unit_weights(seed)
    E = O.stack_errors(W, What)
    rank = min(E.shape)
    vals = [O.importance_ec(E, r) for r in range(0, rank + 3)]
    assert vals[0] == 0.0
    assert all(0.0 <= v <= 1.0 + 1e-15 for v in vals)
    assert all(b >= a - 1e-15 for a, b in zip(vals, vals[1:]))
    assert vals[rank] == pytest.approx(1.0, rel=1e-12) and vals[-1] == pytest.approx(1.0, rel=1e-12)
    # Eckart-Young: what r ranks capture is what the best rank-r approximation keeps
    for r in (1, 4, 8):
        A, B, _ = O.factors_svd(E, r)
        kept = 1.0 - np.linalg.norm(E - A @ B) ** 2 / np.linalg.norm(E) ** 2
        assert O.importance_ec(E, r) == pytest.approx(kept, rel=1e-10)


def test_ec_known_spectrum():
    # a matrix built from a chosen spectrum: the score is a ratio of its squares
    rng = np.random.default_rng(4)
    U, _ = np.linalg.qr(rng.standard_normal((12, 6)))
    V, _ = np.linalg.qr(rng.standard_normal((20, 6)))
    sv = np.array([5.0, 3.0, 2.0, 1.0, 0.5, 0.25])
    M = (U * sv) @ V.T
    for r in range(7):
        assert O.importance_ec(M, r) == pytest.approx(np.sum(sv[:r] ** 2) / np.sum(sv ** 2), rel=1e-12)


def test_ec_from_stored_factors_matches_the_spectrum():
    W, What = _unit_weights(5, d=128, d_outs=(32, 48), G=64)
    E = O.stack_errors(W, What)
    energy = float(np.sum(E ** 2))
    for r in (8, 16):
        A, B, _ = O.factors_svd(E, r)
        A_bits = [O.f64_to_bits(a, "f16") for a in O.split_rows(A, [32, 48])]
        got = O.importance_ec_from_factors(A_bits, O.f64_to_bits(B, "f16"), "f16", energy)
        assert got == pytest.approx(O.importance_ec(E, r), rel=3e-3)      # 16-bit storage of the factors
        # unrounded factors give the score exactly (orthogonal columns and rows)
        exact = float(np.sum(np.sum(A ** 2, axis=0) * np.sum(B ** 2, axis=1)) / energy)
        assert exact == pytest.approx(O.importance_ec(E, r), rel=1e-10)


def test_selection_is_top_k_with_index_order_among_ties():
    scores = [0.3, 0.9, 0.3, 0.5, 0.9, 0.1]
    assert O.select_units(scores, 0).tolist() == [0, 0, 0, 0, 0, 0]
    assert O.select_units(scores, 1).tolist() == [0, 1, 0, 0, 0, 0]
    assert O.select_units(scores, 2).tolist() == [0, 1, 0, 0, 1, 0]
    assert O.select_units(scores, 4).tolist() == [1, 1, 0, 1, 1, 0]
    assert O.select_units(scores, 9).tolist() == [1, 1, 1, 1, 1, 1]
    # brute force: no other subset of size k has a larger score sum
    rng = np.random.default_rng(6)
    s = rng.random(7)
    for k in range(8):
        m = O.select_units(s, k)
        assert int(m.sum()) == k
        best = max((sum(s[list(c)]) for c in itertools.combinations(range(7), k)), default=0.0)
        assert float(s[m.astype(bool)].sum()) == pytest.approx(best, rel=1e-15)
