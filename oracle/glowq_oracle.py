"""CPU oracle for the GlowQ group forward -- TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition the HIP library is checked against.
It is imported by tests/, by __graft_entry__.smoke() and by the cpu_baseline
leg of bench.py, and by nothing else; it shares no code with the HIP path and
never receives a value that the HIP path produced.

What it computes (memory is token-major: X[T][d], W_i[O_i][d], B[r][d],
A_i[O_i][r], R[T][r], Y_i[T][O_i]; the paper writes the same maps in column
form):

  R    = X B^T                                   Sec. 3.3, Eq. 8
  Y_i  = X What_i^T + R A_i^T   (restored unit)  Sec. 3.3, Eq. 9
  Y_i  = X What_i^T             (unit not restored by GlowQ-S, Sec. 3.3)

with What_i = dequant(W_q,i) the stored INT4 weight widened back to the 16-bit
activation type, and the setup that manufactures the stored operands:
round-to-nearest asymmetric INT4 (W4A16, group size G along d; Sec. 4.1),
errors E_i = W_i - What_i stacked by rows (App. A.0), the truncated SVD of the
stack (Sec. 3.1.1, Prop. 1; App. A.1.2) split into balanced factors
(Eq. 7 / Eqs. A.1.9a-c), the least-squares block recovery (Eq. A.1.10), the
QR-reduced randomised variant (Alg. 1), and the importance scores and top-k selection
of GlowQ-S (Eqs. 10-11).

Every operand of the forward is the *stored* 16-bit value widened to float64;
all accumulation is float64; R is never re-rounded.  Pins for every function
are in tests/test_oracle_*.py (nothing here is "parity unpinned").
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence, Tuple

import numpy as np


def _by_row_chunks(fn, n_rows: int, min_rows: int = 256):
    """Apply fn(lo, hi) to row ranges on a few threads (numpy releases the GIL inside its
    loops) and return the results in order.  Rows are independent in everything this is
    used for, so chunking changes no value."""
    workers = max(1, min(16, os.cpu_count() or 1, n_rows // min_rows))
    if workers == 1:
        return [fn(0, n_rows)]
    step = -(-n_rows // workers)
    bounds = [(lo, min(n_rows, lo + step)) for lo in range(0, n_rows, step)]
    with ThreadPoolExecutor(workers) as ex:
        return list(ex.map(lambda b: fn(*b), bounds))

# --------------------------------------------------------------------------
# 16-bit formats: widening and round-to-nearest-even, written out
# --------------------------------------------------------------------------
_FORMATS = {
    # name: (significand bits incl. hidden one, min normal exponent, exponent bits)
    "f16": (11, -14, 5),
    "bf16": (8, -126, 8),
}


def bits_to_f64(bits: np.ndarray, fmt: str) -> np.ndarray:
    """Value of each 16-bit pattern, exactly, as float64 (IEEE binary16 or
    bfloat16: 1 sign bit, e exponent bits, 15 - e fraction bits)."""
    sig, emin, ebits = _FORMATS[fmt]
    fbits = 15 - ebits
    b = np.asarray(bits, dtype=np.uint16).astype(np.int64)
    sign = np.where((b >> 15) & 1, -1.0, 1.0)
    e = (b >> fbits) & ((1 << ebits) - 1)
    f = b & ((1 << fbits) - 1)
    emax_code = (1 << ebits) - 1
    normal = np.ldexp((f + (1 << fbits)).astype(np.float64), (e + emin - 1 - fbits).astype(np.int64))
    subnormal = np.ldexp(f.astype(np.float64), emin - fbits)
    val = np.where(e == 0, subnormal, normal)
    val = np.where((e == emax_code) & (f == 0), np.inf, val)
    val = np.where((e == emax_code) & (f != 0), np.nan, val)
    return sign * val


def f64_to_bits(x: np.ndarray, fmt: str) -> np.ndarray:
    """Round float64 to the 16-bit format, nearest-even, one rounding; returns
    the uint16 bit patterns.  Overflow goes to infinity."""
    sig, emin, ebits = _FORMATS[fmt]
    fbits = 15 - ebits
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    _, e = np.frexp(a)                      # a = m * 2^e, m in [0.5, 1)
    e = np.maximum(e - 1, emin)             # exponent of the leading bit, floored
    quantum_exp = (e - (sig - 1)).astype(np.int64)
    n = np.rint(np.ldexp(a, -quantum_exp))  # integer significand, half-to-even
    # a carry to 2^sig moves to the next binade
    carry = n >= (1 << sig)
    n = np.where(carry, n / 2, n)
    e = np.where(carry, e + 1, e)
    n = np.where(np.isfinite(n), n, 0).astype(np.int64)   # inf / nan are patched below
    is_normal = n >= (1 << (sig - 1))
    code_e = np.where(is_normal, e - emin + 1, 0).astype(np.int64)
    frac = np.where(is_normal, n - (1 << (sig - 1)), n).astype(np.int64)
    emax_code = (1 << ebits) - 1
    overflow = code_e >= emax_code
    code_e = np.where(overflow, emax_code, code_e)
    frac = np.where(overflow, 0, frac)
    out = (code_e << fbits) | frac
    out = np.where(np.isinf(a), emax_code << fbits, out)
    out = np.where(np.isnan(x), (emax_code << fbits) | (1 << (fbits - 1)), out)
    out = out | (np.signbit(x).astype(np.int64) << 15)
    return out.astype(np.uint16)


# --------------------------------------------------------------------------
# W4A16 storage: quantise, pack, unpack, dequantise   (Sec. 4.1: INT4, g128)
# --------------------------------------------------------------------------
def quantize_rtn(W: np.ndarray, G: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Round-to-nearest asymmetric INT4 per (row, group of G along d).

    The paper fixes only "INT4 weights, group size 128" (Sec. 4.1); the reading
    taken here: the group range [lo, hi] is widened to contain 0,
    s = fp16(max((hi - lo) / 15, 2^-14)), z = clamp(rint(-lo / s), 0, 15),
    q = clamp(rint(w / s) + z, 0, 15), rint = half-to-even, divisions on the
    fp16-rounded s in float64.  Returns q uint8 [O][d], and the fp16 bit
    patterns of s and z, each [O][d / G] (z is an integer stored as fp16).
    """
    W = np.asarray(W, dtype=np.float32)
    O, d = W.shape
    assert d % G == 0

    def rows(lo_r, hi_r):
        Wg = W[lo_r:hi_r].reshape(hi_r - lo_r, d // G, G).astype(np.float64)
        lo = np.minimum(Wg.min(axis=2), 0.0)
        hi = np.maximum(Wg.max(axis=2), 0.0)
        s = np.maximum((hi - lo) / 15.0, 2.0 ** -14)
        s_bits = f64_to_bits(s, "f16")
        s_hat = bits_to_f64(s_bits, "f16")
        z = np.clip(np.rint(-lo / s_hat), 0, 15) + 0.0      # (+ 0.0: a zero-point of zero is +0, never -0)
        q = np.clip(np.rint(Wg / s_hat[:, :, None]) + z[:, :, None], 0, 15)
        return q.reshape(hi_r - lo_r, d).astype(np.uint8), s_bits, f64_to_bits(z, "f16")

    parts = _by_row_chunks(rows, O)
    return (np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts]),
            np.concatenate([p[2] for p in parts]))


def pack_int4(q: np.ndarray) -> np.ndarray:
    """Canonical packing: word[o][j] = sum_e q[o][8j + e] << 4e  (element 8j+e
    in bits 4e..4e+3), uint32 [O][d / 8]."""
    q = np.asarray(q, dtype=np.uint8)
    O, d = q.shape
    assert d % 8 == 0 and q.max(initial=0) <= 15
    q8 = q.reshape(O, d // 8, 8).astype(np.uint32)
    word = np.zeros((O, d // 8), dtype=np.uint32)
    for e in range(8):
        word |= q8[:, :, e] << np.uint32(4 * e)
    return word


def unpack_int4(words: np.ndarray) -> np.ndarray:
    """Inverse of pack_int4: uint8 q[O][d] with values 0..15."""
    words = np.asarray(words, dtype=np.uint32)
    O, n = words.shape
    q = np.empty((O, n, 8), dtype=np.uint8)
    for e in range(8):
        q[:, :, e] = (words >> np.uint32(4 * e)) & np.uint32(15)
    return q.reshape(O, n * 8)


def dequant_bits(q: np.ndarray, s_bits: np.ndarray, z_bits: np.ndarray, G: int,
                 act: str) -> np.ndarray:
    """What[o][k] = round_act((q - z) * s): the integer difference and the
    product are exact in float64, so there is exactly one rounding, to the
    activation type.  Returns the uint16 bit patterns [O][d]."""
    q = np.asarray(q)
    s_bits = np.asarray(s_bits)
    z_bits = np.asarray(z_bits)

    def rows(lo, hi):
        s = np.repeat(bits_to_f64(s_bits[lo:hi], "f16"), G, axis=1)
        z = np.repeat(bits_to_f64(z_bits[lo:hi], "f16"), G, axis=1)
        return f64_to_bits((q[lo:hi].astype(np.float64) - z) * s, act)

    return np.concatenate(_by_row_chunks(rows, q.shape[0]))


def dequant(q, s_bits, z_bits, G: int, act: str) -> np.ndarray:
    """dequant_bits widened to float64: the weight the forward multiplies with."""
    bits = dequant_bits(q, s_bits, z_bits, G, act)
    return np.concatenate(_by_row_chunks(lambda lo, hi: bits_to_f64(bits[lo:hi], act),
                                         bits.shape[0]))


# --------------------------------------------------------------------------
# factors of the stacked error  (Sec. 3.1.1, Sec. 3.2, App. A.1)
# --------------------------------------------------------------------------
def stack_errors(W_list: Sequence[np.ndarray], What_list: Sequence[np.ndarray]) -> np.ndarray:
    """E_cat = [E_1; ...; E_m] by rows, E_i = W_i - What_i (App. A.0; the main
    text's Eq. 1 prints the transposed blocks, the appendix and every proof use
    this row stacking, which is what E_cat - A B needs dimensionally)."""
    return np.concatenate(
        [np.asarray(W, np.float64) - np.asarray(Wh, np.float64)
         for W, Wh in zip(W_list, What_list)], axis=0)


def split_rows(A: np.ndarray, d_outs: Sequence[int]) -> List[np.ndarray]:
    """A = [A_1; ...; A_m]: row block i belongs to module i (App. A.0)."""
    out, o = [], 0
    for n in d_outs:
        out.append(A[o:o + n])
        o += n
    return out


def factors_svd(E_cat: np.ndarray, r: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Balanced rank-r factors of the stack from its thin SVD:
    A* = U_r Sigma_r^(1/2), B* = Sigma_r^(1/2) V_r^T (Eqs. A.1.9a-b), the
    Eckart-Young minimiser of ||E_cat - A B||_F (Prop. 1).  Also returns all
    singular values."""
    U, s, Vt = np.linalg.svd(np.asarray(E_cat, np.float64), full_matrices=False)
    root = np.sqrt(s[:r])
    return U[:, :r] * root[None, :], root[:, None] * Vt[:r], s


def ls_block_recovery(E_i: np.ndarray, B: np.ndarray) -> np.ndarray:
    """A_i* = E_i B^T (B B^T)^+  (Eq. A.1.10 / Eq. A.4.4)."""
    B = np.asarray(B, np.float64)
    return np.asarray(E_i, np.float64) @ B.T @ np.linalg.pinv(B @ B.T)


def thin_qr(E: np.ndarray, method: str = "householder") -> Tuple[np.ndarray, np.ndarray]:
    """Thin QR E = Q_e R_e with Q_e^T Q_e = I (Alg. 1, step 1).  "cholesky"
    takes R_e from the Cholesky factor of E^T E (same factorisation up to row
    signs when E has full column rank; O(m d^2) in one matrix product, used for
    the large synthetic shapes whose E is well conditioned)."""
    E = np.asarray(E, np.float64)
    if method == "householder":
        return np.linalg.qr(E, mode="reduced")
    if method == "none":
        # no reduction: Q_e = I, R_e = E (the randomised steps then run on the stack itself;
        # same estimator, used where a QR of the stack would dominate a test's run time)
        return None, E
    if method == "cholesky":
        L = np.linalg.cholesky(E.T @ E)
        Re = L.T
        from scipy.linalg import solve_triangular

        Qe = solve_triangular(Re, E.T, trans="T", lower=False).T
        return Qe, Re
    raise ValueError(method)


def factors_alg1(E_cat: np.ndarray, r: int, p: int, q: int, Omega: np.ndarray,
                 sigma_x_diag: Optional[np.ndarray] = None,
                 qr: str = "householder") -> Tuple[np.ndarray, np.ndarray]:
    """QR-reduced randomised SVD (Alg. 1) for a diagonal input covariance.

    Omega is the d x (r+p) Gaussian test matrix (drawn by the caller).  Steps in
    the algorithm's order: thin QR of the stack; core M = R_e Sigma_x^(1/2);
    sketch Y = M Omega with q power steps Y <- M (M^T Y); orthonormal basis Q;
    small SVD of Q^T M; lift U = Q U~; truncate and balance; lift back,
    A* = Q_e A^*, B* = B^* Sigma_x^(-1/2).  With sigma_x_diag None the
    covariance is the identity (the unweighted problem of Sec. 3.1.1).
    """
    E_cat = np.asarray(E_cat, np.float64)
    d = E_cat.shape[1]
    assert Omega.shape == (d, r + p)
    Qe, Re = thin_qr(E_cat, qr)
    if sigma_x_diag is None:
        root = np.ones(d)
    else:
        root = np.sqrt(np.asarray(sigma_x_diag, np.float64))
    M = Re * root[None, :]
    Y = M @ np.asarray(Omega, np.float64)
    for _ in range(q):
        Y = M @ (M.T @ Y)
    Q, _ = np.linalg.qr(Y, mode="reduced")
    Ut, s, Vt = np.linalg.svd(Q.T @ M, full_matrices=False)
    U = Q @ Ut
    rs = np.sqrt(s[:r])
    A_hat = U[:, :r] * rs[None, :]
    B_hat = rs[:, None] * Vt[:r]
    inv_root = np.where(root > 0, 1.0 / np.where(root > 0, root, 1.0), 0.0)
    A = A_hat if Qe is None else Qe @ A_hat
    return A, B_hat * inv_root[None, :]


# --------------------------------------------------------------------------
# the forward  (Sec. 3.3, Eqs. 8-9)
# --------------------------------------------------------------------------
def shared_proj(X_bits: np.ndarray, B_bits: np.ndarray, act: str) -> np.ndarray:
    """R[t][j] = sum_k X[t][k] B[j][k], float64, not re-rounded (Eq. 8)."""
    return bits_to_f64(X_bits, act) @ bits_to_f64(B_bits, act).T


def module_forward(module: dict, X_bits: np.ndarray, R: Optional[np.ndarray],
                   G: int, act: str) -> np.ndarray:
    """Y_i[t][o] = sum_k X[t][k] What_i[o][k] (+ sum_j R[t][j] A_i[o][j] when R
    is given), float64 (Eq. 9).  With R None the second sum is absent."""
    q = unpack_int4(module["wq"])
    What = dequant(q, module["scales"], module["zeros"], G, act)
    Y = bits_to_f64(X_bits, act) @ What.T
    if R is not None:
        Y = Y + R @ bits_to_f64(module["A"], act).T
    return Y


def group_forward(unit: dict, restore: bool = True) -> List[np.ndarray]:
    """One unit (input-sharing group or solo module): R once, then every module
    (Sec. 3.3).  A unit that is not restored, or has rank 0, skips Eq. 8 and the
    correction term of Eq. 9 altogether."""
    act, G = unit["act"], unit["G"]
    R = None
    if restore and unit["r"] > 0:
        R = shared_proj(unit["X"], unit["B"], act)
    return [module_forward(m, unit["X"], R, G, act) for m in unit["modules"]]


def block_forward(units: Sequence[dict], restore_mask: Sequence[int]) -> List[List[np.ndarray]]:
    """GlowQ-S: the correction is applied only to the selected units (Sec. 3.3)."""
    return [group_forward(u, bool(f)) for u, f in zip(units, restore_mask)]


def layerwise_forward(unit: dict) -> List[np.ndarray]:
    """The layer-wise comparison point of the latency study (Sec. 4.3): nothing is
    shared, every module i computes a projection of its own, R_i = X B_i^T, and then
    Y_i = X What_i^T + R_i A_i^T.  B_i is the module's own right factor `module["B"]`
    when the unit was set up layer-wise (`build_unit_layerwise`); a module without one
    takes the unit's shared B, which must reproduce `group_forward` exactly (Prop. 1:
    the shared projection serves every module)."""
    act, G = unit["act"], unit["G"]
    out = []
    for m in unit["modules"]:
        B_i = m["B"] if "B" in m else unit["B"]
        R_i = shared_proj(unit["X"], B_i, act) if unit["r"] > 0 else None
        out.append(module_forward(m, unit["X"], R_i, G, act))
    return out


# --------------------------------------------------------------------------
# importance of a unit and the GlowQ-S selection  (Sec. 3.3, Eqs. 10-11)
# --------------------------------------------------------------------------
def importance_ner(W_list: Sequence[np.ndarray], What_list: Sequence[np.ndarray]) -> float:
    """g_ner(u) = ||E_u||_F^2 / ||W_u||_F^2 over all modules of the unit (Eq. 11);
    E_u is the stacked error, W_u the stacked full-precision weight."""
    e = sum(float(np.sum((np.asarray(W, np.float64) - np.asarray(Wh, np.float64)) ** 2))
            for W, Wh in zip(W_list, What_list))
    w = sum(float(np.sum(np.asarray(W, np.float64) ** 2)) for W in W_list)
    return e / w


def importance_ec(M_u: np.ndarray, r: int) -> float:
    """g_ec(u) = sum_{j<=r} sigma_j(M_u)^2 / ||M_u||_F^2 (Eq. 10): the share of the
    aligned error's energy that r ranks capture.  M_u is the stacked error after
    covariance alignment; with Sigma_x = I (the reading the workloads use) M_u = E_u."""
    sv = np.linalg.svd(np.asarray(M_u, np.float64), compute_uv=False)
    return float(np.sum(sv[:r] ** 2) / np.sum(sv ** 2))


def importance_ec_from_factors(A_bits_list: Sequence[np.ndarray], B_bits: np.ndarray, act: str,
                               error_energy: float) -> float:
    """The same share read off the STORED balanced factors: the columns of A = U S^(1/2)
    and the rows of B = S^(1/2) V^T are orthogonal with ||a_j||^2 = ||b_j||^2 = sigma_j
    (Eqs. A.1.9a-b), so sum_j ||a_j||^2 ||b_j||^2 = sum_j sigma_j^2.  This is what can be
    evaluated where only the stored operands are at hand; it differs from importance_ec
    by the 16-bit rounding of the factors."""
    A = np.concatenate([bits_to_f64(a, act) for a in A_bits_list], axis=0)
    B = bits_to_f64(B_bits, act)
    return float(np.sum(np.sum(A ** 2, axis=0) * np.sum(B ** 2, axis=1)) / error_energy)


def select_units(scores: Sequence[float], k: int) -> np.ndarray:
    """GlowQ-S: the k units with the highest score are restored (Sec. 3.3); among equal
    scores the unit with the lower index comes first.  Returns the 0/1 mask."""
    scores = np.asarray(scores, np.float64)
    order = np.argsort(-scores, kind="stable")
    mask = np.zeros(len(scores), np.uint8)
    mask[order[:max(0, min(int(k), len(scores)))]] = 1
    return mask


# --------------------------------------------------------------------------
# setup of one unit from full-precision weights
# --------------------------------------------------------------------------
def build_unit(W_list: Sequence[np.ndarray], X_bits: np.ndarray, r: int, G: int,
               act: str, method: str = "svd", Omega: Optional[np.ndarray] = None,
               p: int = 16, q: int = 2, qr: str = "cholesky") -> dict:
    """Quantise each module, factorise the stacked error, round the factors to
    the activation type, and return the stored operands of the unit."""
    modules, What_list = [], []
    for W in W_list:
        qv, s_bits, z_bits = quantize_rtn(W, G)
        modules.append(dict(wq=pack_int4(qv), scales=s_bits, zeros=z_bits,
                            d_out=W.shape[0]))
        What_list.append(dequant(qv, s_bits, z_bits, G, act))
    d = W_list[0].shape[1]
    if r > 0:
        E_cat = stack_errors(W_list, What_list)
        if method == "svd":
            A, B, _ = factors_svd(E_cat, r)
        elif method == "alg1":
            A, B = factors_alg1(E_cat, r, p, q, Omega, None, qr=qr)
        else:
            raise ValueError(method)
        for m, A_i in zip(modules, split_rows(A, [W.shape[0] for W in W_list])):
            m["A"] = f64_to_bits(A_i, act)
        B_bits = f64_to_bits(B, act)
    else:
        for m in modules:
            m["A"] = np.zeros((m["d_out"], 0), np.uint16)
        B_bits = np.zeros((0, d), np.uint16)
    return dict(X=np.asarray(X_bits, np.uint16), B=B_bits, modules=modules,
                act=act, G=G, r=r, d_in=d, T=X_bits.shape[0])


def build_unit_layerwise(W_list: Sequence[np.ndarray], X_bits: np.ndarray, r: int, G: int,
                         act: str) -> dict:
    """The same quantised modules with layer-wise factors: each error block E_i gets the
    truncated SVD of its own, E_i ~ A_i B_i (the independent per-layer correction the
    paper compares against, Sec. 2 and Sec. 4.3), both factors rounded to the activation
    type.  The unit carries no shared B."""
    if r <= 0:
        raise ValueError("layer-wise factors need r > 0")
    modules = []
    for W in W_list:
        if r > min(W.shape):
            raise ValueError("rank above the size of an error block")
        qv, s_bits, z_bits = quantize_rtn(W, G)
        What = dequant(qv, s_bits, z_bits, G, act)
        A_i, B_i, _ = factors_svd(stack_errors([W], [What]), r)
        modules.append(dict(wq=pack_int4(qv), scales=s_bits, zeros=z_bits, d_out=W.shape[0],
                            A=f64_to_bits(A_i, act), B=f64_to_bits(B_i, act)))
    d = W_list[0].shape[1]
    return dict(X=np.asarray(X_bits, np.uint16), B=np.zeros((0, d), np.uint16), modules=modules,
                act=act, G=G, r=r, d_in=d, T=X_bits.shape[0])
