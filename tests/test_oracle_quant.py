"""Pins for the oracle's fp16 conversion, quantizer, packer and dequantizer (Section 3.2).

None of these re-types the oracle's formula: they check it against numpy's independent
float16, hand-derived byte fixtures, invariants the definition implies, and lossless cases.
"""
import numpy as np
import pytest

import oracle
from conftest import golden_path

BITS = (2, 4, 8)


def qmax(b):
    return (1 << (b - 1)) - 1


# ------------------------------------------------------------------ fp16 conversion
def test_f16_to_f32_exhaustive_against_numpy():
    h = np.arange(65536, dtype=np.uint16)
    ref = h.view(np.float16).astype(np.float32)
    got = np.array([oracle.f16_bits_to_f32(int(v)) for v in h], dtype=np.float32)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))


def test_f32_to_f16_against_numpy_including_ties_and_subnormals():
    rng = np.random.default_rng(1)
    vals = [0.0, -0.0, 1.0, 65504.0, 65519.9, 65520.0, 1e-8, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
            3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11,
            2047.5, 2048.5, 1e6, -1e6]
    vals += list(rng.standard_normal(20000) * 0.01)
    vals += list(np.exp(rng.uniform(-20, 12, 20000)) * rng.choice([-1, 1], 20000))
    # exact ties between neighbouring halves
    h = rng.integers(0, 0x7bff, 5000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals += list((lo + hi) / 2)
    vals = np.array(vals, dtype=np.float32)
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f32_to_f16_bits(v) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)


# ------------------------------------------------------------------ pack / unpack
def _fixtures():
    out = []
    for line in open(golden_path("pack_rows.txt")):
        if line.startswith("#") or not line.strip():
            continue
        b, codes, hexs = [s.strip() for s in line.split("|")]
        out.append((int(b), np.array(codes.split(), dtype=np.int8), bytes.fromhex(hexs)))
    return out


def test_pack_matches_hand_derived_rows():
    fx = _fixtures()
    assert sorted(b for b, _, _ in fx) == [2, 4, 8]
    for b, codes, raw in fx:
        got = oracle.pack(codes[None, :], b)
        assert got.tobytes() == raw, f"bits={b}"
        assert np.array_equal(oracle.unpack(np.frombuffer(raw, np.uint8)[None, :], 32, b)[0], codes)


@pytest.mark.parametrize("b", BITS)
def test_pack_single_element_positions(b):
    """Every code value at every position of a 16-byte word: exactly the expected bits are set."""
    per_word = 128 // b
    for pos in range(per_word):
        for code in range(-qmax(b), qmax(b) + 1):
            q = np.zeros((1, per_word), np.int8)
            q[0, pos] = code
            word = int.from_bytes(oracle.pack(q, b).tobytes(), "little")
            zero_word = int.from_bytes(oracle.pack(np.zeros((1, per_word), np.int8), b).tobytes(), "little")
            field = (word >> (pos * b)) & ((1 << b) - 1)
            assert field == code + (1 << (b - 1))
            mask = ((1 << b) - 1) << (pos * b)
            assert (word & ~mask) == (zero_word & ~mask)


@pytest.mark.parametrize("b", BITS)
def test_pack_unpack_round_trip_random(b):
    rng = np.random.default_rng(b)
    q = rng.integers(-qmax(b), qmax(b) + 1, size=(7, 192)).astype(np.int8)
    p = oracle.pack(q, b)
    assert p.shape == (7, 192 * b // 8)
    assert np.array_equal(oracle.unpack(p, 192, b), q)


# ------------------------------------------------------------------ quantizer invariants
@pytest.mark.parametrize("b", BITS)
@pytest.mark.parametrize("g", (32, 64, 128))
def test_quant_error_at_most_half_a_step_and_max_element_hits_qmax(b, g):
    rng = np.random.default_rng(10 * b + g)
    w = (rng.standard_normal((24, 4 * g)) * 0.02).astype(np.float32)
    w[3, :g] = 0.0                       # an all-zero group
    w[5, g:2 * g] *= 1e-3                # a small-magnitude group
    q, s = oracle.quantize(w, b, g)
    sf = s.view(np.float16).astype(np.float64)
    wq = q.astype(np.float64) * np.repeat(sf, g, axis=1)
    err = np.abs(w.astype(np.float64) - wq)
    assert np.all(err <= np.repeat(sf, g, axis=1) / 2 * (1 + 2.0 ** -22))
    assert np.all(np.abs(q) <= qmax(b))
    qg = np.abs(q.reshape(24, 4, g)).max(axis=2)
    wg = np.abs(w.reshape(24, 4, g)).max(axis=2)
    normal = sf >= 2.0 ** -14            # fp16 subnormal scales are too coarse for the next two claims
    assert normal.sum() >= 24 * 4 - 3
    assert np.all(qg[normal] == qmax(b)), "the largest element of a group must map to +-qmax"
    assert np.all(qg[wg > 0] >= 1)
    assert np.all(q.reshape(24, 4, g)[wg == 0] == 0) and np.all(s[wg == 0] == 0)
    # scale is the max-abs over the integer range, within one fp16 step above
    ideal = wg / qmax(b)
    nz = wg > 0
    assert np.all(sf[nz] >= ideal[nz] * (1 - 2.0 ** -23))
    assert np.all(sf[normal] <= ideal[normal] * (1 + 2.0 ** -9))


@pytest.mark.parametrize("b", BITS)
def test_quant_lossless_when_weights_are_scale_times_integers(b):
    """W = s0 * integers with s0 a power of two and a +-qmax in every group -> exact codes back."""
    rng = np.random.default_rng(b)
    g = 32
    ints = rng.integers(-qmax(b), qmax(b) + 1, size=(9, 3 * g))
    ints[:, ::g] = qmax(b) * rng.choice([-1, 1], size=(9, 3))
    s0 = 2.0 ** -7
    w = (ints * s0).astype(np.float32)
    q, s = oracle.quantize(w, b, g)
    assert np.array_equal(q, ints.astype(np.int8))
    assert np.all(s.view(np.float16) == np.float16(s0))
    wd = oracle.dequant(oracle.pack(q, b), s, 3 * g, b, g)
    assert np.array_equal(wd, w)


@pytest.mark.parametrize("b", BITS)
def test_quant_idempotent_on_its_own_output(b):
    rng = np.random.default_rng(100 + b)
    g = 64
    w = (rng.standard_normal((16, 2 * g)) * 0.02).astype(np.float32)
    q, s = oracle.quantize(w, b, g)
    wd = oracle.dequant(oracle.pack(q, b), s, 2 * g, b, g)
    q2, s2 = oracle.quantize(wd, b, g)
    assert np.array_equal(q2, q) and np.array_equal(s2, s)


def test_quant_ties_round_to_even():
    # scale exactly 1/8 (absmax 7/8 at 4 bits); w/s = k + 0.5 must go to the even neighbour
    g = 32
    w = np.zeros((1, g), np.float32)
    w[0, 0] = 7 / 8
    w[0, 1:7] = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5], np.float32) / 8
    q, s = oracle.quantize(w, 4, g)
    assert s.view(np.float16)[0, 0] == np.float16(0.125)
    assert list(q[0, :7]) == [7, 0, 2, 2, 0, -2, -2]


def test_int2_is_ternary_and_int8_range():
    rng = np.random.default_rng(7)
    w = rng.standard_normal((8, 64)).astype(np.float32)
    q2, _ = oracle.quantize(w, 2, 32)
    assert set(np.unique(q2)) <= {-1, 0, 1}
    q8, _ = oracle.quantize(w, 8, 32)
    assert q8.min() >= -127 and q8.max() <= 127


def test_scale_bumped_up_instead_of_clamping():
    # absmax/qmax that rounds DOWN in fp16: without the one-step bump the max element would need |q| > qmax
    g = 32
    found = 0
    rng = np.random.default_rng(3)
    for _ in range(2000):
        a = np.float32(rng.uniform(0.01, 0.1))
        s32 = np.float32(a / np.float32(7))
        sh = np.float16(s32)
        if np.float32(sh) * np.float32(7) < a:
            found += 1
            w = np.zeros((1, g), np.float32)
            w[0, 0] = a
            q, s = oracle.quantize(w, 4, g)
            assert q[0, 0] == 7
            assert s[0, 0] == sh.view(np.uint16) + 1
    assert found > 100


def _round_fraction_to_f32(fr):
    """The float32 nearest to an exact rational (ties to even), found by exact comparison."""
    from fractions import Fraction
    c = np.float32(float(fr))
    cands = [np.nextafter(c, np.float32(-np.inf)), c, np.nextafter(c, np.float32(np.inf))]
    best = min(cands, key=lambda v: (abs(Fraction(float(v)) - fr), int(np.float32(v).view(np.uint32)) & 1))
    return np.float32(best)


@pytest.mark.parametrize("w_bits,s_bits,code", [
    # (fp32 bits of w, fp16 bits of the group's scale s, the code the definition gives).
    # w / s in exact arithmetic lies just off n + 1/2; the correctly rounded fp32 quotient stays on that side,
    # while w * (1/s) (reciprocal rounded to fp32 first) crosses to the other neighbour:
    (0x3d3627ff, 0x2797, 1),   # w = 0.0444717..., s = 0.0296478...: quotient just below 1.5 -> 1 (product gives 2)
    (0x3e786c01, 0x28c7, 7),   # w = 0.2425995..., s = 0.0373230...: quotient just above 6.5 -> 7 (product gives 6)
    (0x3d756fff, 0x2194, 5),   # w = 0.0599213..., s = 0.0108948...: quotient just below 5.5 -> 5 (product gives 6)
    (0x3c5ee401, 0x1a31, 5),   # w = 0.0136042..., s = 0.0030231...: quotient just above 4.5 -> 5 (product gives 4)
])
def test_codes_come_from_an_fp32_division_not_from_a_reciprocal_multiply(w_bits, s_bits, code):
    """The reading of Section 3.2 taken here fixes q = rint(w / scale) with an fp32 DIVISION. Groups are built
    whose scale is a chosen fp16 value (largest element = 7 * s, exactly representable, so absmax / 7 == s with
    no bump) and that hold one element whose quotient sits next to a rounding boundary."""
    from fractions import Fraction
    w = np.array([w_bits], np.uint32).view(np.float32)[0]
    s = np.array([s_bits], np.uint16).view(np.float16)[0]
    sf = np.float32(s)
    # independent derivation of the expected code with exact rationals
    quot = _round_fraction_to_f32(Fraction(float(w)) / Fraction(float(sf)))
    assert int(np.rint(quot)) == code
    recip = _round_fraction_to_f32(1 / Fraction(float(sf)))
    prod = _round_fraction_to_f32(Fraction(float(w)) * Fraction(float(recip)))
    assert int(np.rint(prod)) != code, "the case must separate the two formulas"
    g = 32
    grp = np.zeros((1, g), np.float32)
    grp[0, 0] = np.float32(7) * sf
    grp[0, 1] = w
    grp[0, 2] = -w
    q, sc = oracle.quantize(grp, 4, g)
    assert sc[0, 0] == s_bits
    assert list(q[0, :3]) == [7, code, -code]


# ------------------------------------------------------------------ dequant closed form
@pytest.mark.parametrize("b", BITS)
def test_dequant_is_scale_times_code_exactly(b):
    rng = np.random.default_rng(50 + b)
    g = 32
    q = rng.integers(-qmax(b), qmax(b) + 1, size=(5, 4 * g)).astype(np.int8)
    s = rng.uniform(1e-4, 4e-2, size=(5, 4)).astype(np.float16)
    wd = oracle.dequant(oracle.pack(q, b), s.view(np.uint16), 4 * g, b, g)
    ref = (np.repeat(s.astype(np.float64), g, axis=1) * q).astype(np.float32)  # exact: 11-bit x 8-bit
    assert np.array_equal(wd, ref)


def test_rejects_bad_arguments():
    w = np.zeros((2, 48), np.float32)
    with pytest.raises(ValueError):
        oracle.quantize(w, 3, 16)
    with pytest.raises(ValueError):
        oracle.quantize(w, 4, 32)   # 48 % 32 != 0
