"""Pins for the oracle's codecs (paper Section 2 and Section 3.1).  No GPU."""
import decimal
import math
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def golden():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].split()
        if len(line) >= 3:
            out[line[0]] = (float(line[1]), float(line[2]))
    return out


def dec_ln(x: float, prec: int = 60) -> decimal.Decimal:
    decimal.getcontext().prec = prec
    return decimal.Decimal(x).ln()


def round_to(comp, value: decimal.Decimal):
    """Round an exact decimal to the nearest float of the component type by comparing the
    two neighbouring floats exactly (independent of any libm)."""
    approx = comp(float(value))
    cands = [np.nextafter(approx, comp(-np.inf)), approx, np.nextafter(approx, comp(np.inf))]
    errs = [abs(decimal.Decimal(float(c)) - value) for c in cands]
    return cands[int(np.argmin(errs))]


def test_paper_printed_values(oracle):
    g = golden()
    # Section 2: 3 + 2 pi i and 3 + 4 pi i stand for the same real number exp(3)
    z = np.array([3 + 2j * math.pi, 3 + 4j * math.pi], dtype=np.complex128)
    x = oracle.from_goom(z)
    v, tol = g["equal_representations_exp3"]
    assert x[0] == x[1] and abs(x[0] - v) <= tol
    # odd multiples are negative
    x = oracle.from_goom(np.array([3 + 1j * math.pi, 3 + 3j * math.pi, 3 - 1j * math.pi], dtype=np.complex128))
    assert np.all(x < 0) and np.allclose(x, -math.exp(3))
    # Section 3.1 footnote: finite floor for Float32 components
    v, tol = g["float32_log_zero_floor"]
    assert abs(oracle.floor_value(np.float32) - v) <= tol
    snn, tol2 = g["float32_smallest_normal"]
    assert abs(np.finfo(np.float32).tiny - snn) <= tol2
    assert abs(oracle.floor_value(np.float32) - 2 * math.log(float(np.finfo(np.float32).tiny))) < 1e-4
    assert abs(oracle.floor_value(np.float64) - 2 * math.log(np.finfo(np.float64).tiny)) < 1e-9
    # the floor exponentiates to zero at component precision
    assert oracle.from_goom(np.array([oracle.floor_value(np.float32)], dtype=np.complex64))[0] == 0.0
    assert oracle.from_goom(np.array([oracle.floor_value(np.float64)], dtype=np.complex128))[0] == 0.0


def test_zero_and_special_values(oracle):
    x = np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf], dtype=np.float32)
    z = oracle.to_goom(x)
    assert z[0].real == -np.inf and z[0].imag == 0.0  # zero is a non-negative GOOM (Section 2)
    assert z[1].real == -np.inf and z[1].imag == 0.0
    assert z[2] == 0 and z[3].real == 0.0 and z[3].imag == np.float32(np.pi)
    assert z[4].real == np.inf and z[4].imag == 0 and z[5].real == np.inf and z[5].imag == np.float32(np.pi)
    zf = oracle.to_goom(x[:2], zero_floor=True)
    assert np.all(zf.real == np.float32(oracle.floor_value(np.float32))) and np.all(zf.imag == 0)
    assert np.isnan(oracle.to_goom(np.array([np.nan], dtype=np.float64))[0].real)
    # imaginary constant is the component type's nearest value to pi
    assert oracle.to_goom(np.array([-2.0], dtype=np.float64))[0].imag == math.pi
    assert oracle.to_goom(np.array([-2.0], dtype=np.float32))[0].imag == np.float32(math.pi)


@pytest.mark.parametrize("comp", [np.float32, np.float64])
def test_encode_is_correctly_rounded(oracle, comp):
    rng = np.random.default_rng(7)
    xs = np.concatenate([
        rng.standard_normal(300), np.exp(rng.uniform(-80, 80, 300)) * rng.choice([-1, 1], 300),
        [1.0, -1.0, 2.0, 0.5, math.e, 1e-30, -3e30, float(np.finfo(comp).tiny), float(np.finfo(comp).max)],
        [float(np.finfo(comp).smallest_subnormal) * 3],
    ]).astype(comp)
    z = oracle.to_goom(xs)
    for x, zz in zip(xs, z):
        want = round_to(comp, dec_ln(abs(float(x))))
        assert zz.real == want, (x, zz.real, want)
        assert zz.imag == (comp(math.pi) if x < 0 else 0)


def test_encode_powers_of_two_closed_form(oracle):
    # log(2^k) = k log 2, to the last bit
    ks = np.arange(-120, 121)
    x = np.ldexp(np.float32(1.0), ks).astype(np.float32)
    z = oracle.to_goom(x)
    decimal.getcontext().prec = 60
    ln2 = decimal.Decimal(2).ln()
    for k, zz in zip(ks, z):
        assert zz.real == round_to(np.float32, ln2 * int(k))


@pytest.mark.parametrize("comp,ctype", [(np.float32, np.complex64), (np.float64, np.complex128)])
def test_decode_is_correctly_rounded_and_signed(oracle, comp, ctype):
    rng = np.random.default_rng(11)
    re = rng.uniform(-60, 60, 400).astype(comp)
    sg = rng.integers(0, 2, 400)
    z = np.empty(400, dtype=ctype)
    z.real = re
    z.imag = sg * comp(math.pi)
    x = oracle.from_goom(z)
    decimal.getcontext().prec = 60
    for r, s, xx in zip(re, sg, x):
        want = round_to(comp, decimal.Decimal(float(r)).exp())
        assert abs(xx) == want and (xx < 0) == bool(s)


def test_round_trip_error_bound(oracle):
    # exp of the GOOM recovers the real value to within |log|x|| * eps (the log is rounded once)
    rng = np.random.default_rng(3)
    x = (np.exp(rng.uniform(-80, 80, 20000)) * rng.choice([-1.0, 1.0], 20000)).astype(np.float32)
    back = oracle.from_goom(oracle.to_goom(x))
    eps = np.finfo(np.float32).eps
    rel = np.abs(back.astype(np.float64) / x.astype(np.float64) - 1)
    bound = (np.abs(np.log(np.abs(x.astype(np.float64)))) + 1) * eps
    assert np.all(rel <= bound)
    assert np.all(np.sign(back) == np.sign(x))


def test_dynamic_range_survives(oracle):
    # Table 1: Complex64 GOOMs span exp(+-1e38); products of such numbers are additions (Example 1)
    big = np.array([[3e38 + 0j]], dtype=np.complex64)
    one = np.array([[0 + 0j]], dtype=np.complex64)
    re, sg = oracle.lmme(big, one)
    assert re[0, 0] == np.float64(np.float32(3e38)) and sg[0, 0] == 0
    small = np.array([[-3e38 + 1j * np.float32(np.pi)]], dtype=np.complex64)
    re, sg = oracle.lmme(small, one)
    assert re[0, 0] == np.float64(np.float32(-3e38)) and sg[0, 0] == 1


def test_split_accepts_any_representative(oracle):
    z = np.array([1 + 0j, 1 + 1j * math.pi, 1 + 2j * math.pi, 1 - 3j * math.pi, 1 + 3.1j], dtype=np.complex128)
    re, sg = oracle.split(z)
    assert list(sg) == [0, 1, 0, 1, 1] and np.all(re == 1.0)
