"""Pins for the oracle's factor generator (stacked SVD, balanced split, block
recovery, QR-reduced randomised SVD).  Every check is a closed form the paper
states: Eckart-Young residual (App. A.1.2), balance (Lemma A.1.4), least-squares
block recovery (Eq. A.1.10), reduction to the core (Alg. 1 / App. A.3)."""
import numpy as np
import pytest

from oracle import glowq_oracle as O


def _stack(seed=0, d_outs=(40, 24, 56), d=32):
    rng = np.random.default_rng(seed)
    E = [rng.standard_normal((o, d)) * np.linspace(2.0, 0.1, d)[None, :] for o in d_outs]
    return E, np.concatenate(E, axis=0)


def test_row_stacking_and_split_are_inverse():
    rng = np.random.default_rng(1)
    W = [rng.standard_normal((5, 8)), rng.standard_normal((3, 8))]
    Wh = [np.zeros((5, 8)), np.ones((3, 8))]
    E = O.stack_errors(W, Wh)
    assert E.shape == (8, 8)
    assert np.array_equal(E[:5], W[0]) and np.array_equal(E[5:], W[1] - 1.0)
    parts = O.split_rows(E, [5, 3])
    assert np.array_equal(parts[0], E[:5]) and np.array_equal(parts[1], E[5:])


@pytest.mark.parametrize("r", [1, 4, 16])
def test_eckart_young_residual_equals_tail_energy(r):
    _, E = _stack()
    A, B, s = O.factors_svd(E, r)
    assert A.shape == (E.shape[0], r) and B.shape == (r, E.shape[1])
    res = np.linalg.norm(E - A @ B, "fro") ** 2
    assert res == pytest.approx(np.sum(s[r:] ** 2), rel=1e-10)
    # no other rank-r product does better: perturbing the factors raises the residual
    rng = np.random.default_rng(2)
    for _ in range(5):
        A2 = A + 1e-3 * rng.standard_normal(A.shape)
        B2 = B + 1e-3 * rng.standard_normal(B.shape)
        assert np.linalg.norm(E - A2 @ B2, "fro") ** 2 >= res


def test_balanced_split():
    _, E = _stack(3)
    r = 8
    A, B, s = O.factors_svd(E, r)
    Sr = np.diag(s[:r])
    assert np.allclose(A.T @ A, Sr, atol=1e-12)
    assert np.allclose(B @ B.T, Sr, atol=1e-12)
    # singular values come from an independent route: eigenvalues of E^T E
    ev = np.sort(np.linalg.eigvalsh(E.T @ E))[::-1]
    assert np.allclose(s[:r] ** 2, ev[:r], rtol=1e-10)


def test_block_recovery_equals_row_block():
    Es, E = _stack(4)
    r = 8
    A, B, _ = O.factors_svd(E, r)
    blocks = O.split_rows(A, [e.shape[0] for e in Es])
    for E_i, A_i in zip(Es, blocks):
        assert np.allclose(O.ls_block_recovery(E_i, B), A_i, atol=1e-10)
    # and it is the least-squares solution: the normal equations hold
    A0 = O.ls_block_recovery(Es[0], B)
    assert np.allclose(A0 @ (B @ B.T), Es[0] @ B.T, atol=1e-10)


def test_full_rank_factors_reproduce_the_stack():
    Es, E = _stack(5, d_outs=(20, 20), d=16)
    A, B, _ = O.factors_svd(E, 16)
    assert np.allclose(A @ B, E, atol=1e-12)


def test_shared_B_is_at_least_as_good_as_any_common_B():
    # Prop. 1: among products with ONE right factor, the stacked SVD is optimal;
    # the per-module optimum with its own B_i can only be better or equal
    Es, E = _stack(6)
    r = 4
    A, B, s = O.factors_svd(E, r)
    shared = sum(np.linalg.norm(E_i - A_i @ B, "fro") ** 2
                 for E_i, A_i in zip(Es, O.split_rows(A, [e.shape[0] for e in Es])))
    assert shared == pytest.approx(np.sum(s[r:] ** 2), rel=1e-10)
    per_module = 0.0
    for E_i in Es:
        si = np.linalg.svd(E_i, compute_uv=False)
        per_module += np.sum(si[r:] ** 2)
    assert per_module <= shared + 1e-12
    # a B taken from one module alone is worse for the group than the shared one
    _, B0, _ = O.factors_svd(Es[0], r)
    alt = sum(np.linalg.norm(E_i - O.ls_block_recovery(E_i, B0) @ B0, "fro") ** 2 for E_i in Es)
    assert alt >= shared - 1e-12


@pytest.mark.parametrize("qr", ["householder", "cholesky"])
def test_thin_qr(qr):
    _, E = _stack(7)
    Q, R = O.thin_qr(E, qr)
    d = E.shape[1]
    assert Q.shape == E.shape and R.shape == (d, d)
    assert np.allclose(Q.T @ Q, np.eye(d), atol=1e-9)
    assert np.allclose(Q @ R, E, atol=1e-10)
    assert np.allclose(np.tril(R, -1), 0.0)


@pytest.mark.parametrize("qr", ["householder", "cholesky", "none"])
def test_alg1_identity_covariance_matches_exact_svd(qr):
    # a decaying spectrum with a clear gap after r: with p = 8, q = 2 the sketch
    # captures the leading subspace to rounding, so the products agree
    rng = np.random.default_rng(8)
    m, d, r = 96, 40, 6
    U, _ = np.linalg.qr(rng.standard_normal((m, d)))
    V, _ = np.linalg.qr(rng.standard_normal((d, d)))
    s = np.concatenate([np.linspace(10, 5, r), 1e-3 * np.ones(d - r)])
    E = (U * s) @ V.T
    A0, B0, _ = O.factors_svd(E, r)
    Omega = rng.standard_normal((d, r + 8))
    A1, B1 = O.factors_alg1(E, r, 8, 2, Omega, None, qr=qr)
    assert np.allclose(A1 @ B1, A0 @ B0, atol=1e-6)
    # balanced in the identity metric
    assert np.allclose(A1.T @ A1, B1 @ B1.T, atol=1e-8)


def test_alg1_weighted_objective_is_the_whitened_optimum():
    # Prop. 3: the minimiser of ||(E - AB) Sigma^(1/2)||_F is the truncated SVD of
    # E Sigma^(1/2); with the full sketch (r + p = d) Alg. 1 is exact
    rng = np.random.default_rng(9)
    m, d, r = 60, 24, 5
    E = rng.standard_normal((m, d))
    sig = np.exp(rng.standard_normal(d))
    Omega = rng.standard_normal((d, d))
    A, B = O.factors_alg1(E, r, d - r, 1, Omega, sig)
    root = np.sqrt(sig)
    got = np.linalg.norm((E - A @ B) * root[None, :], "fro") ** 2
    sw = np.linalg.svd(E * root[None, :], compute_uv=False)
    assert got == pytest.approx(np.sum(sw[r:] ** 2), rel=1e-9)
    # and it beats the unweighted factors in the weighted metric
    A0, B0, _ = O.factors_svd(E, r)
    assert got <= np.linalg.norm((E - A0 @ B0) * root[None, :], "fro") ** 2 + 1e-12


def test_alg1_error_within_randomised_bound():
    # Halko-type expectation bound (App. A.4): with oversampling p >= 2 the
    # Frobenius error is at most (1 + r/(p-1))^(1/2) * tail; checked with slack 2
    rng = np.random.default_rng(10)
    m, d, r, p = 200, 64, 8, 8
    E = rng.standard_normal((m, d)) * (1.0 / np.arange(1, d + 1))[None, :]
    s = np.linalg.svd(E, compute_uv=False)
    tail = np.sqrt(np.sum(s[r:] ** 2))
    Omega = rng.standard_normal((d, r + p))
    A, B = O.factors_alg1(E, r, p, 0, Omega, None)
    err = np.linalg.norm(E - A @ B, "fro")
    assert tail * (1 - 1e-12) <= err <= 2.0 * np.sqrt(1 + r / (p - 1)) * tail
