"""Pins for the oracle's storage arithmetic: 16-bit formats, INT4 packing,
RTN quantiser, single-rounding dequantisation (W4A16, Sec. 4.1).

Each check compares the oracle with something that is not the oracle: library
casts (numpy binary16, torch bfloat16), exact integer arithmetic on the bit
patterns, a hand-worked example, or closed-form bounds.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import glowq_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- formats
def test_widen_all_f16_patterns_against_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = O.bits_to_f64(bits, "f16")
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok])
    assert np.array_equal(np.signbit(ref[ok]), np.signbit(got[ok]))


def test_widen_all_bf16_patterns_against_torch():
    bits = np.arange(65536, dtype=np.uint16)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    ref = t.to(torch.float64).numpy()
    got = O.bits_to_f64(bits, "bf16")
    ok = ~np.isnan(ref)
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    assert np.array_equal(ref[ok], got[ok])


def _random_doubles(n, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n) * np.exp(rng.uniform(-40, 12, n))
    return x


def test_round_f16_against_numpy_cast():
    x = _random_doubles(200000, 1)
    # add exact ties and subnormal-range values
    ties = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25,
                     65504.0, 65519.99, 65520.0, 1e9, -2.0 ** -14 + 2.0 ** -26, 0.0, -0.0])
    x = np.concatenate([x, ties, -ties])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(O.f64_to_bits(x, "f16"), ref)


def test_round_bf16_against_torch_cast_of_f32_values():
    # values that are exactly float32, so torch's f32 -> bf16 cast is one rounding
    x = _random_doubles(200000, 2).astype(np.float32)
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.3895313892515355e38, 1e39,
                     2.0 ** -133, 3 * 2.0 ** -134, 0.0], dtype=np.float64)
    with np.errstate(over="ignore"):
        x = np.concatenate([x, ties.astype(np.float32), -ties.astype(np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.f64_to_bits(x.astype(np.float64), "bf16"), ref)


def test_round_trip_is_identity_on_every_finite_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    for fmt in ("f16", "bf16"):
        v = O.bits_to_f64(bits, fmt)
        fin = np.isfinite(v)
        assert np.array_equal(O.f64_to_bits(v[fin], fmt), bits[fin])


# ---------------------------------------------------------------- packing
def test_pack_hand_example_and_every_nibble_position():
    q = np.array([[1, 2, 3, 4, 5, 6, 7, 8]], dtype=np.uint8)
    assert O.pack_int4(q)[0, 0] == 0x87654321
    for e in range(8):
        for v in range(16):
            q = np.zeros((1, 8), np.uint8)
            q[0, e] = v
            w = O.pack_int4(q)
            assert int(w[0, 0]) == v << (4 * e)
            assert np.array_equal(O.unpack_int4(w), q)


def test_pack_unpack_round_trip_random(naive):
    rng = np.random.default_rng(3)
    q = rng.integers(0, 16, size=(37, 264), dtype=np.uint8)
    w = O.pack_int4(q)
    assert w.shape == (37, 33) and w.dtype == np.uint32
    assert np.array_equal(O.unpack_int4(w), q)
    assert np.array_equal(naive.unpack(w), q)          # C oracle reads the same layout
    # word j holds elements 8j..8j+7 of its own row only
    q2 = q.copy()
    q2[5, 17] ^= 1
    diff = np.argwhere(O.pack_int4(q2) != w)
    assert diff.tolist() == [[5, 2]]


# ---------------------------------------------------------------- quantiser
def _read_golden():
    d = {}
    with open(os.path.join(GOLDEN, "rtn_worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = v
    return d


def test_rtn_worked_example():
    g = _read_golden()
    w = np.array([[-0.7, -0.5, -0.3, -0.1, 0.1, 0.3, 0.5, 0.8]], dtype=np.float32)
    q, s_bits, z_bits = O.quantize_rtn(w, 8)
    assert int(s_bits[0, 0]) == int(g["scale_bits"][0], 16)
    assert int(z_bits[0, 0]) == int(g["zero_bits"][0], 16)
    assert q[0].tolist() == [int(v) for v in g["q"]]
    assert int(O.pack_int4(q)[0, 0]) == int(g["word"][0], 16)
    what = O.dequant(q, s_bits, z_bits, 8, "f16")
    den = 2.0 ** int(g["what_den_log2"][0])
    assert what[0].tolist() == [int(v) / den for v in g["what_num"]]


def test_rtn_bounds_and_ranges():
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((64, 512)) * 0.02).astype(np.float32)
    W[3, 128:256] = 0.0                      # a zero-range group
    W[4, 0:128] = np.abs(W[4, 0:128])        # an all-positive group
    for G in (64, 128):
        q, s_bits, z_bits = O.quantize_rtn(W, G)
        s = np.repeat(O.bits_to_f64(s_bits, "f16"), G, axis=1)
        z = np.repeat(O.bits_to_f64(z_bits, "f16"), G, axis=1)
        assert q.min() >= 0 and q.max() <= 15
        assert np.all((z >= 0) & (z <= 15) & (z == np.rint(z)))
        assert np.all(s >= 2.0 ** -14)        # normal fp16, never zero
        # the zero-point is an unsigned 4-bit integer stored as binary16: its patterns are
        # those of 0.0 .. 15.0, the sign bit never set (a one-sided positive group has z = +0)
        assert set(np.unique(z_bits)) <= {int(np.float16(v).view(np.uint16)) for v in range(16)}
        assert z_bits[4, 0] == 0 and z_bits[3, 128 // G] == 0
        what = O.dequant(q, s_bits, z_bits, G, "f16")
        unclamped = (q > 0) & (q < 15)
        err = np.abs(W.astype(np.float64) - what)
        bound = s / 2 + np.abs(what) * 2.0 ** -11
        assert np.all(err[unclamped] <= bound[unclamped] * (1 + 1e-12))
        assert np.all(what[3, 128:256] == 0.0)
        # every group uses (almost) the whole code range
        qg = q.reshape(64, -1, G)
        assert np.median(qg.max(axis=2) - qg.min(axis=2)) >= 14


# ---------------------------------------------------------------- dequant
def _dequant_by_integers(q: int, z: int, s_bits: int, fmt: str) -> Fraction:
    """Independent formulation: s = m * 2^e from its fp16 fields; (q - z) * m is
    an integer that is rounded to the format's significand width by integer
    arithmetic (ties to even); result returned as an exact fraction."""
    e = (s_bits >> 10) & 31
    f = s_bits & 1023
    if e == 0:
        m, ex = f, -24
    else:
        m, ex = f + 1024, e - 25
    n = (q - z) * m
    if n == 0:
        return Fraction(0)
    sig, emin = {"f16": (11, -14), "bf16": (8, -126)}[fmt]
    sign = -1 if n < 0 else 1
    n = abs(n)
    drop = max(n.bit_length() - sig, (emin - (sig - 1)) - ex)
    if drop > 0:
        half = 1 << (drop - 1)
        rem = n & ((1 << drop) - 1)
        n >>= drop
        if rem > half or (rem == half and (n & 1)):
            n += 1
        ex += drop
    return sign * Fraction(n) * Fraction(2) ** ex


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_dequant_single_rounding_all_codes(fmt):
    # all 1024 fractions at one exponent, plus small, large and subnormal scales;
    # every (q, z) pair for each of them: one row per (scale, z), 16 columns q = 0..15
    scales = [0x2000 + f for f in range(1024)] + [0x0400, 0x0401, 0x07FF, 0x3C00, 0x5640,
                                                 0x0001, 0x03FF, 0x1234, 0x2E66]
    rows = [(sb, z) for sb in scales for z in range(16)]
    q = np.tile(np.arange(16, dtype=np.uint8), (len(rows), 1))
    s_bits = np.array([[sb] for sb, _ in rows], dtype=np.uint16)
    z_bits = O.f64_to_bits(np.array([[float(z)] for _, z in rows]), "f16")
    got = O.dequant(q, s_bits, z_bits, 16, fmt)
    for i, (sb, z) in enumerate(rows):
        for qv in range(16):
            assert Fraction(float(got[i, qv])) == _dequant_by_integers(qv, z, sb, fmt), \
                (hex(sb), z, qv)


def test_dequant_matches_c_oracle_bitwise(naive):
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((48, 384)) * 0.02).astype(np.float32)
    q, s_bits, z_bits = O.quantize_rtn(W, 128)
    mod = dict(wq=O.pack_int4(q), scales=s_bits, zeros=z_bits)
    for fmt in ("f16", "bf16"):
        a = O.dequant(q, s_bits, z_bits, 128, fmt)
        b = naive.dequant(mod, 128, fmt)
        assert np.array_equal(a, b)
        # the value is representable in the format: re-rounding changes nothing
        assert np.array_equal(O.bits_to_f64(O.f64_to_bits(a, fmt), fmt), a)


def test_dequant_group_index_runs_along_input_dim():
    # scales differ per group: element k must use group k // G of ITS row
    q = np.full((2, 256), 9, np.uint8)
    s = O.f64_to_bits(np.array([[1.0, 2.0], [4.0, 8.0]]), "f16")
    z = O.f64_to_bits(np.array([[8.0, 7.0], [6.0, 5.0]]), "f16")
    w = O.dequant(q, s, z, 128, "f16")
    assert np.all(w[0, :128] == 1.0) and np.all(w[0, 128:] == 4.0)
    assert np.all(w[1, :128] == 12.0) and np.all(w[1, 128:] == 32.0)


# --------------------------------------------------------------------------
# the row-chunk helper: the threaded branch returns what the single-chunk branch returns
# --------------------------------------------------------------------------
@pytest.mark.parametrize("n_rows", [1, 255, 256, 511, 512, 1000, 1025, 4097, 5000])
def test_row_chunks_cover_every_row_once_in_order(n_rows):
    parts = O._by_row_chunks(lambda lo, hi: (lo, hi), n_rows)
    assert parts[0][0] == 0 and parts[-1][1] == n_rows
    for (lo, hi), (lo2, _) in zip(parts, parts[1:]):
        assert lo < hi == lo2
    if n_rows >= 512 and (os.cpu_count() or 1) > 1:
        assert len(parts) > 1            # the threaded branch really ran


@pytest.mark.parametrize("act", ["f16", "bf16"])
def test_threaded_rows_equal_single_chunk_rows(act):
    """quantize_rtn / dequant_bits / dequant on 1536 + 40 rows (several chunks, a ragged
    last one) equal, row for row, the same functions applied to slices short enough to
    take the single-chunk branch."""
    rng = np.random.default_rng(11)
    n_rows, d, G = 1576, 256, 64
    W = (rng.standard_normal((n_rows, d)) * 0.02).astype(np.float32)
    q, s_bits, z_bits = O.quantize_rtn(W, G)
    wb = O.dequant_bits(q, s_bits, z_bits, G, act)
    wf = O.dequant(q, s_bits, z_bits, G, act)
    assert q.shape == (n_rows, d) and s_bits.shape == (n_rows, d // G) and wb.shape == (n_rows, d)
    for lo in range(0, n_rows, 200):                 # 200 < 256: one chunk, no threads
        hi = min(n_rows, lo + 200)
        q1, s1, z1 = O.quantize_rtn(W[lo:hi], G)
        assert np.array_equal(q[lo:hi], q1)
        assert np.array_equal(s_bits[lo:hi], s1) and np.array_equal(z_bits[lo:hi], z1)
        assert np.array_equal(wb[lo:hi], O.dequant_bits(q1, s1, z1, G, act))
        assert np.array_equal(wf[lo:hi], O.dequant(q1, s1, z1, G, act))
