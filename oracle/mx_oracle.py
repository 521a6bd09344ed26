"""Oracle of the microscaling variant of the group forward: MXFP4 weights and MXFP8
activations in the main product, the low-rank correction unchanged.

TEST INFRASTRUCTURE ONLY: plain numpy in float64, slow and obviously correct; only tests/,
__graft_entry__.smoke() and bench.py's baseline / check legs may use it.  It shares no code
with the HIP path.

What the paper fixes: GlowQ is layered on weight-only MXFP4 ("microscaling-style formats in
which weights are first normalised within a small block and then encoded using low-bit
floating-point codes ... following the OCP MX specification", App. "Compatibility Across
Quantization Datatypes"), and on a W4A8 setting (main results table, Sec. 4).  The formats
themselves are those of the public OCP Microscaling Formats (MX) specification v1.0,
restated here:
  block      32 consecutive elements along the input dimension share one scale
  scale      E8M0: an 8-bit exponent code c, value 2^(c - 127), c = 255 is NaN (never made)
  MXFP4      element E2M1: sign, 2 exponent bits (bias 1), 1 fraction bit; magnitudes
             0, 0.5, 1, 1.5, 2, 3, 4, 6; no infinities, no NaN
  MXFP8      element E4M3: sign, 4 exponent bits (bias 7), 3 fraction bits; largest finite
             448 (S.1111.110); S.1111.111 is NaN; subnormals m / 8 * 2^-6
  conversion shared exponent = floor(log2(max |v|)) - emax_elem (emax_elem = 2 for E2M1, 8 for
             E4M3), clamped to [-127, 127]; every element is v / 2^shared rounded to the
             element format, ties to even, magnitudes above the largest finite value clamped
             to it.
Readings where the specification leaves a choice: a block of zeros gets the scale code 127
(scale 1) and zero elements; non-finite inputs are not supported.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

from . import glowq_oracle as O

BLOCK = 32
FORMATS = {
    #          exponent bits, fraction bits, bias, emax of the largest finite value, largest finite value
    "e2m1": dict(ebits=2, mbits=1, bias=1, emax=2, vmax=6.0),
    "e4m3": dict(ebits=4, mbits=3, bias=7, emax=8, vmax=448.0),
}


def element_values(fmt: str) -> np.ndarray:
    """Value of every code of an element format (float64; NaN where the code is NaN)."""
    f = FORMATS[fmt]
    n = 1 << (1 + f["ebits"] + f["mbits"])
    out = np.empty(n, np.float64)
    for c in range(n):
        sign = -1.0 if c >> (f["ebits"] + f["mbits"]) else 1.0
        e = (c >> f["mbits"]) & ((1 << f["ebits"]) - 1)
        m = c & ((1 << f["mbits"]) - 1)
        if e == 0:
            v = m / (1 << f["mbits"]) * 2.0 ** (1 - f["bias"])
        else:
            v = (1 + m / (1 << f["mbits"])) * 2.0 ** (e - f["bias"])
        if fmt == "e4m3" and e == 15 and m == 7:
            v = np.nan
        out[c] = sign * v
    return out


def scale_values(codes: np.ndarray) -> np.ndarray:
    """E8M0: 2^(code - 127)."""
    return np.ldexp(1.0, np.asarray(codes, np.int64) - 127)


def round_to_element(v: np.ndarray, fmt: str) -> np.ndarray:
    """Codes of v rounded to the element format: nearest, ties to even, saturating."""
    f = FORMATS[fmt]
    v = np.asarray(v, np.float64)
    a = np.abs(v)
    emin = 1 - f["bias"]
    _, ex = np.frexp(np.where(a > 0, a, 1.0))              # a = m 2^ex, m in [0.5, 1)
    e = np.maximum(ex - 1, emin)                            # binade of a, not below the subnormal one
    quantum = np.ldexp(1.0, e - f["mbits"])
    q = np.rint(a / quantum) * quantum                      # exact scaling, one rounding, half to even
    q = np.minimum(q, f["vmax"])
    # encode the rounded magnitude
    _, qx = np.frexp(np.where(q > 0, q, 1.0))
    qe = np.maximum(qx - 1, emin)
    is_sub = q < 2.0 ** emin
    frac = np.where(is_sub, q / 2.0 ** emin, q / np.ldexp(1.0, qe) - 1.0) * (1 << f["mbits"])
    code = np.where(is_sub, 0, qe + f["bias"]).astype(np.int64) << f["mbits"] | frac.astype(np.int64)
    code = np.where(q == 0, 0, code)
    sign = (np.signbit(v) & (q != 0)).astype(np.int64) << (f["ebits"] + f["mbits"])
    return (code | sign).astype(np.uint8)


def mx_quantize(V: np.ndarray, fmt: str) -> Tuple[np.ndarray, np.ndarray]:
    """Rows of V [n][d] to MX blocks along d: element codes uint8 [n][d] and scale codes
    uint8 [n][d / 32]."""
    f = FORMATS[fmt]
    V = np.asarray(V, np.float64)
    n, d = V.shape
    assert d % BLOCK == 0 and np.all(np.isfinite(V))
    Vb = V.reshape(n, d // BLOCK, BLOCK)
    amax = np.max(np.abs(Vb), axis=2)
    _, ex = np.frexp(np.where(amax > 0, amax, 1.0))
    shared = np.clip(ex - 1 - f["emax"], -127, 127)
    shared = np.where(amax > 0, shared, 0)
    codes = round_to_element(Vb / np.ldexp(1.0, shared)[:, :, None], fmt)
    return codes.reshape(n, d), (shared + 127).astype(np.uint8)


def mx_dequant(codes: np.ndarray, scales: np.ndarray, fmt: str) -> np.ndarray:
    """element value times block scale, exactly, float64 [n][d]."""
    vals = element_values(fmt)[np.asarray(codes, np.int64)]
    return vals * np.repeat(scale_values(scales), BLOCK, axis=1)


def pack_fp4(codes: np.ndarray) -> np.ndarray:
    """uint32 [n][d / 8]: element 8j + e of a row in bits 4e .. 4e + 3 of word j."""
    return O.pack_int4(codes)


def mx_group_forward(unit: dict, restore: bool = True):
    """Y_i = Xq What_i^T + R A_i^T with R = X B^T (Sec. 3.3, Eqs. 8-9): the main product on
    the dequantised MXFP8 activations Xq and MXFP4 weights What_i, the correction from the
    16-bit activations X and the 16-bit factors, as in the W4A16 path."""
    act = unit["act"]
    X = O.bits_to_f64(unit["X"], act)
    xc, xs = mx_quantize(X, "e4m3")
    Xq = mx_dequant(xc, xs, "e4m3")
    R = None
    if restore and unit["r"] > 0:
        R = X @ O.bits_to_f64(unit["B"], act).T
    out = []
    for m in unit["modules"]:
        What = mx_dequant(m["codes"], m["scales"], "e2m1")
        Y = Xq @ What.T
        if R is not None:
            Y = Y + R @ O.bits_to_f64(m["A"], act).T
        out.append(Y)
    return out


def build_unit_mx(W_list: Sequence[np.ndarray], X_bits: np.ndarray, r: int, act: str) -> dict:
    """MXFP4 weights of every module, and the balanced rank-r factors of the stacked error
    E = W - dequant (Eqs. A.1.9a-b) rounded to the activation type."""
    modules, What = [], []
    for W in W_list:
        codes, scales = mx_quantize(W, "e2m1")
        modules.append(dict(codes=codes, scales=scales, d_out=W.shape[0]))
        What.append(mx_dequant(codes, scales, "e2m1"))
    d = W_list[0].shape[1]
    if r > 0:
        A, B, _ = O.factors_svd(O.stack_errors(W_list, What), r)
        for m, A_i in zip(modules, O.split_rows(A, [W.shape[0] for W in W_list])):
            m["A"] = O.f64_to_bits(A_i, act)
        B_bits = O.f64_to_bits(B, act)
    else:
        for m in modules:
            m["A"] = np.zeros((m["d_out"], 0), np.uint16)
        B_bits = np.zeros((0, d), np.uint16)
    return dict(X=np.asarray(X_bits, np.uint16), B=B_bits, modules=modules, act=act, r=r,
                d_in=d, T=X_bits.shape[0])
