"""Pins for the oracle's LMME, chain scan and affine recurrence (paper Sections 3.2, 4.1,
4.3 and Appendix C).  Brute force uses exact rational arithmetic or numpy long double; no
GPU and no call back into the routine under test."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import digamma

import synthetic_inputs as si


def goom_of(x, ctype=np.complex128):
    """GOOM of a real array by the definition (Section 3.1), with numpy only."""
    x = np.asarray(x, dtype=np.float64)
    z = np.empty(x.shape, dtype=ctype)
    with np.errstate(divide="ignore"):
        z.real = np.log(np.abs(x))
    z.imag = np.where(x < 0, np.pi, 0.0)
    return z


def exact_product(a, b):
    """Exact rational matrix product of two float arrays."""
    n, d = a.shape
    m = b.shape[1]
    fa = [[Fraction(float(v)) for v in row] for row in a]
    fb = [[Fraction(float(v)) for v in row] for row in b]
    return [[sum(fa[i][j] * fb[j][k] for j in range(d)) for k in range(m)] for i in range(n)]


def assert_matches_real(re, sg, exact, rtol):
    for i, row in enumerate(exact):
        for k, v in enumerate(row):
            if v == 0:
                assert re[i, k] == -np.inf
                continue
            want = math.log(abs(v.numerator)) - math.log(v.denominator) if isinstance(v, Fraction) else math.log(abs(v))
            assert abs(re[i, k] - want) <= rtol * max(1.0, abs(want)), (i, k, re[i, k], want)
            assert bool(sg[i, k]) == (v < 0)


def test_lmme_matches_exact_rational_products(oracle):
    rng = np.random.default_rng(5)
    for (n, d, m) in [(1, 1, 1), (3, 5, 2), (8, 8, 8), (4, 17, 9)]:
        a = rng.standard_normal((n, d))
        b = rng.standard_normal((d, m))
        a[0, 0] = 0.0  # a zero entry is the GOOM (-inf, +)
        re, sg = oracle.lmme(goom_of(a), goom_of(b))
        assert_matches_real(re, sg, exact_product(a, b), 1e-12)


def test_lmme_transposed_operands_would_fail(oracle):
    # guards against a swapped index in the oracle: A B != B A and != A^T B in general
    rng = np.random.default_rng(6)
    a = rng.standard_normal((4, 4))
    b = rng.standard_normal((4, 4))
    re, sg = oracle.lmme(goom_of(a), goom_of(b))
    want = a @ b
    assert np.allclose(np.where(sg == 1, -1, 1) * np.exp(re), want, rtol=1e-12)
    assert not np.allclose(want, b @ a) and not np.allclose(want, a.T @ b)


def test_lmme_exp1000_dot_product_example(oracle):
    # Example 2: a_j = b_j = exp(1000): every term is 2000 and the dot product is log(d) above it
    gold = dict(l.split("#")[0].split()[:2] for l in open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")) if l.strip() and not l.startswith("#"))
    term = float(gold["dot_product_term_log"])
    for d in (1, 7, 64):
        a = np.full((1, d), 1000.0 + 0j)
        b = np.full((d, 1), 1000.0 + 0j)
        re, sg = oracle.lmme(a, b)
        assert abs(re[0, 0] - (term + math.log(d))) < 1e-12 and sg[0, 0] == 0


def test_lmme_scaling_identity(oracle):
    # Section 3.2, eq. 12: shifting rows of A' by r_i and columns of B' by c_k shifts the result
    # by r_i + c_k exactly; shifting column j of A' up and row j of B' down changes nothing.
    rng = np.random.default_rng(8)
    n, d, m = 5, 6, 4
    A = goom_of(rng.standard_normal((n, d)))
    B = goom_of(rng.standard_normal((d, m)))
    re0, sg0 = oracle.lmme(A, B)
    r = rng.integers(-2000, 2000, n).astype(np.float64)
    c = rng.integers(-2000, 2000, m).astype(np.float64)
    A2 = A + r[:, None]
    B2 = B + c[None, :]
    re1, sg1 = oracle.lmme(A2, B2)
    assert np.array_equal(sg0, sg1)
    assert np.allclose(re1, re0 + r[:, None] + c[None, :], rtol=0, atol=1e-9)
    t = rng.integers(-500, 500, d).astype(np.float64)
    re2, sg2 = oracle.lmme(A + t[None, :], B - t[:, None])
    assert np.array_equal(sg0, sg2) and np.allclose(re2, re0, rtol=0, atol=1e-9)


def test_lmme_identity_permutation_and_scalar(oracle):
    rng = np.random.default_rng(9)
    X = goom_of(rng.standard_normal((6, 6)))
    eye = goom_of(np.eye(6))
    re, sg = oracle.lmme(eye, X)
    assert np.array_equal(re, X.real) and np.array_equal(sg, (X.imag != 0).astype(np.uint8))
    perm = np.eye(6)[rng.permutation(6)]
    re, sg = oracle.lmme(goom_of(perm), X)
    assert np.array_equal(re, (perm @ X.real)) or np.allclose(re, perm @ X.real)
    # d = 1: multiplication is addition of GOOMs (Example 1): logs add, signs xor
    a = np.array([[2.5 + 1j * np.pi]])
    b = np.array([[-7.25 + 1j * np.pi]])
    re, sg = oracle.lmme(a, b)
    assert re[0, 0] == -4.75 and sg[0, 0] == 0
    # all-zero row gives zeros, not NaN
    Z = goom_of(np.zeros((2, 6)))
    re, sg = oracle.lmme(Z, X)
    assert np.all(re == -np.inf) and np.all(sg == 0)


def test_lmme_kappa_is_cancellation_factor(oracle):
    a = goom_of(np.array([[1.0, 1.0, -1.999]]))
    b = goom_of(np.array([[1.0], [1.0], [1.0]]))
    re, sg, kap = oracle.lmme(a, b, return_kappa=True)
    assert abs(kap[0, 0] - 3.999 / 0.001) < 1e-6 * kap[0, 0]


def brute_chain_longdouble(mats, init=None):
    """P_t = M_t P_{t-1} in numpy long double, no logs (brute force)."""
    T, d, _ = mats.shape
    out = []
    p = None if init is None else init.astype(np.longdouble)
    for t in range(T):
        mt = mats[t].astype(np.longdouble)
        if p is None:
            p = mt.copy()
        else:
            q = np.zeros((d, p.shape[1]), dtype=np.longdouble)
            for j in range(d):
                q += mt[:, j:j + 1] * p[j:j + 1, :]
            p = q
        out.append(p.copy())
    return np.stack(out)


def test_scan_config1_matches_brute_force(oracle):
    # T = 256 chain of 8 x 8 N(0, 1) matrices: log-norms reach ~250, inside long double range
    x = si.normal_chain(si.BASE_SEED + 1, 256, 8)
    Z = oracle.to_goom(x)
    re, sg, kap = oracle.scan(Z, return_kappa=True)
    # brute force on exactly the reals the GOOMs stand for
    xr = np.where(oracle.split(Z)[1] == 1, -1.0, 1.0) * np.exp(Z.real.astype(np.float64))
    P = brute_chain_longdouble(xr)
    want_re = np.log(np.abs(P)).astype(np.float64)
    # error grows with the chain's accumulated rounding times the cancellation of each entry
    tol = 1e-9 * np.maximum(1.0, np.abs(want_re)) * np.maximum(1.0, kap / 1e3)
    assert np.all(np.abs(re - want_re) <= tol)
    assert np.array_equal(sg.astype(bool), P < 0)
    assert re[0].tolist() == Z[0].real.astype(np.float64).tolist()  # P_1 = M_1
    assert 200 < np.max(re[-1]) < 300


def test_scan_worked_example_and_order(oracle):
    # Appendix C, scan without resets: outputs X_0, A_1 X_0, A_2 A_1 X_0, A_3 A_2 A_1 X_0
    rng = np.random.default_rng(12)
    A = rng.standard_normal((3, 4, 4))
    X0 = rng.standard_normal((4, 4))
    re, sg = oracle.scan(goom_of(A), init=goom_of(X0))
    want = [A[0] @ X0, A[1] @ A[0] @ X0, A[2] @ A[1] @ A[0] @ X0]
    for t in range(3):
        got = np.where(sg[t] == 1, -1, 1) * np.exp(re[t])
        assert np.allclose(got, want[t], rtol=1e-11, atol=0)
    wrong = X0 @ A[0] @ A[1] @ A[2]  # newer factor on the right would be a different matrix
    assert not np.allclose(np.where(sg[2] == 1, -1, 1) * np.exp(re[2]), wrong)
    # rectangular initial state (a vector u_0, Section 4.2.2)
    u0 = rng.standard_normal((4, 1))
    re, sg = oracle.scan(goom_of(A), init=goom_of(u0))
    assert re.shape == (3, 4, 1)
    assert np.allclose(np.where(sg[2] == 1, -1, 1) * np.exp(re[2]), A[2] @ A[1] @ A[0] @ u0, rtol=1e-11)


def test_scan_split_with_init_is_associative(oracle):
    x = si.normal_chain(si.BASE_SEED + 2, 64, 8)
    Z = oracle.to_goom(x)
    re, sg = oracle.scan(Z)
    re1, sg1 = oracle.scan(Z[:40])
    re2, sg2 = oracle.scan(Z[40:], init=(re1[-1], sg1[-1]))
    assert np.array_equal(sg[40:], sg2) and np.allclose(re[40:], re2, rtol=1e-13, atol=1e-12)
    # streaming form gives the same states
    st = oracle.ScanStream(8)
    a_re, a_sg = st.advance(Z[:40], sample_t=[0, 39])
    b_re, b_sg = st.advance(Z[40:], sample_t=[23])
    assert np.array_equal(a_re[1], re[39]) and np.array_equal(b_re[0], re[63]) and np.array_equal(b_sg[0], sg[63])


def test_scan_growth_rate_closed_form(oracle):
    # For i.i.d. N(0,1) d x d factors the top Lyapunov exponent is (ln 2 + psi(d/2)) / 2,
    # because |G u|^2 is chi-square with d degrees of freedom for a unit vector u.
    d, T = 8, 6000
    x = si.normal_chain(si.BASE_SEED + 3, T, d)
    st = oracle.ScanStream(d, scaled=True)
    re, sg = st.advance(oracle.to_goom(x), sample_t=[T - 1])
    lam = 0.5 * (math.log(2) + digamma(d / 2))
    var = 0.25 * 2 * (1.0 / (d / 2))  # ~ var of 0.5 ln chi2_d is trigamma(d/2)/4 <~ 1/(2d) * 2
    rate = 0.5 * np.log(np.sum(np.exp(2 * (re[0] - re[0].max())))) / T + re[0].max() / T
    assert abs(rate - lam) < 5 * math.sqrt(var / T) + 5.0 / T
    assert abs(lam - 0.9746) < 1e-3


def test_scaled_oracle_agrees_with_definitional(oracle):
    for d, T in [(8, 300), (16, 200), (64, 48)]:
        Z = oracle.to_goom(si.normal_chain(si.BASE_SEED + 4, T, d))
        re, sg, kap = oracle.scan(Z, return_kappa=True)
        st = oracle.ScanStream(d, scaled=True)
        sre, ssg, skap = st.advance(Z, sample_t=list(range(T)), return_kappa=True)
        ok = kap < 1e6
        assert np.array_equal(sg[ok], ssg[ok])
        assert np.all(np.abs(re - sre)[ok] <= 1e-9 * np.maximum(1.0, np.abs(re[ok])) * np.maximum(1, kap[ok]))
        assert np.allclose(kap[1:][ok[1:]], skap[1:][ok[1:]], rtol=1e-6)
    # with an initial state
    Z = oracle.to_goom(si.normal_chain(si.BASE_SEED + 5, 100, 8))
    S0 = oracle.to_goom(si.normal_init(si.BASE_SEED + 5, 8, 3))
    re, sg = oracle.scan(Z, init=S0)
    st = oracle.ScanStream(8, m=3, init=S0, scaled=True)
    sre, ssg = st.advance(Z, sample_t=list(range(100)))
    assert np.array_equal(sg, ssg) and np.allclose(re, sre, rtol=1e-10, atol=1e-9)


def test_scaled_oracle_on_the_first_16384_steps_of_the_long_chain(oracle):
    # The second chain oracle (real mantissas with per-column power-of-two exponents) serves the full-size
    # and the d > 128 parity tests, so it is held against the definitional signed log-sum-exp chain
    # (Section 3.2, the LMME definition; Section 4.1, the chain) where that one can still be run: the first
    # 16 384 steps of the long 64 x 64 chain (log-magnitudes reach 3.4e4, far past double range as reals),
    # at 65 sampled prefixes, every entry; and on short chains of 128 x 128 and 256 x 256 matrices.
    for d, T, every in [(64, 16384, 256), (128, 96, 8), (256, 24, 4)]:
        Z = oracle.to_goom(si.normal_chain(si.BASE_SEED * 10 + 2, T, d))
        samples = sorted(set(list(range(every - 1, T, every)) + [0, T - 1]))
        a = oracle.ScanStream(d)
        b = oracle.ScanStream(d, scaled=True)
        re, sg, kap = a.advance(Z, sample_t=samples, return_kappa=True)
        sre, ssg, skap = b.advance(Z, sample_t=samples, return_kappa=True)
        ok = kap < 1e6
        assert ok.mean() > 0.999
        assert np.array_equal(sg[ok], ssg[ok])
        # both walk the same chain in double: they differ by rounding that the cancellation factor magnifies,
        # accumulated over the steps (a random walk: sqrt(T) units of 2^-53 on log-magnitudes of size |re|)
        bound = 2.0 ** -52 * math.sqrt(T) * 8 * np.maximum(1.0, np.abs(re)) * np.maximum(1.0, kap)
        assert np.all(np.abs(re - sre)[ok] <= bound[ok]), float((np.abs(re - sre) / bound)[ok].max())
        assert np.allclose(kap[1:][ok[1:]], skap[1:][ok[1:]], rtol=1e-5)
        if d == 64:
            assert re.max() > 3.0e4  # about 2.07 per step


# ------------------------------------------------------------------------------ affine

def brute_affine(A, b, h0):
    h = h0.astype(np.longdouble)
    out = []
    for t in range(A.shape[0]):
        h = (A[t].astype(np.longdouble) * h[None, :]).sum(axis=1) + b[t].astype(np.longdouble)
        out.append(h.copy())
    return np.stack(out)


def test_affine_matches_brute_force(oracle):
    A, b = si.recurrence_inputs(si.BASE_SEED + 6, 3, 200, 8)
    h0 = np.zeros(8)
    re, sg, kap = oracle.affine_scan(oracle.to_goom(A), oracle.to_goom(b), return_kappa=True)
    for q in range(3):
        Ar = oracle.from_goom(oracle.to_goom(A[q]).astype(np.complex128))
        br = oracle.from_goom(oracle.to_goom(b[q]).astype(np.complex128))
        want = brute_affine(Ar, br, h0)
        got = np.where(sg[q] == 1, -1.0, 1.0) * np.exp(re[q])
        assert np.allclose(got, want.astype(np.float64), rtol=1e-8, atol=0)


def test_affine_degenerate_cases(oracle):
    rng = np.random.default_rng(21)
    d, T = 5, 12
    b = rng.standard_normal((T, d))
    # A == 0: h_t = b_t
    re, sg = oracle.affine_scan(goom_of(np.zeros((T, d, d))), goom_of(b))
    assert np.allclose(re, np.log(np.abs(b))) and np.array_equal(sg.astype(bool), b < 0)
    # b == 0, h_0 != 0: the plain chain applied to a vector
    A = rng.standard_normal((T, d, d))
    h0 = rng.standard_normal(d)
    re, sg = oracle.affine_scan(goom_of(A), goom_of(np.zeros((T, d))), h0=goom_of(h0))
    re2, sg2 = oracle.scan(goom_of(A), init=goom_of(h0[:, None]))
    assert np.allclose(re, re2[:, :, 0], rtol=1e-13) and np.array_equal(sg, sg2[:, :, 0])
    # time-invariant scalar recurrence: geometric series h_t = b (1 - a^t) / (1 - a)
    a, bb = 0.5, 3.0
    re, sg = oracle.affine_scan(goom_of(np.full((T, 1, 1), a)), goom_of(np.full((T, 1), bb)))
    want = bb * (1 - a ** np.arange(1, T + 1)) / (1 - a)
    assert np.allclose(np.exp(re[:, 0]), want, rtol=1e-13) and np.all(sg == 0)


def test_scaled_exponentiation_of_states(oracle):
    # Section 4.3, eq. 27: c = max Re, scaled = exp(x' - c + 2): values within [-e^2, e^2], the largest
    # entry exactly e^2 in magnitude, ratios of entries preserved, a common shift of the logs cancels
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 12)) * np.exp(rng.uniform(-30, 30, (7, 12)))
    z = oracle.to_goom(x)
    s, c = oracle.scaled_exp(z)
    assert np.allclose(c, np.log(np.abs(x).max(axis=1)), rtol=1e-15)
    assert np.allclose(np.abs(s).max(axis=1), math.e ** 2, rtol=1e-14)
    assert np.allclose(s, x / np.abs(x).max(axis=1, keepdims=True) * math.e ** 2, rtol=1e-12)
    shifted = z + 5000.0  # far outside double range as reals
    s2, c2 = oracle.scaled_exp(shifted)
    assert np.allclose(s2, s, rtol=1e-12) and np.allclose(c2, c + 5000.0)
    # the worked numbers: logs (0, -1, 1 + i pi) give c = 1 and (e, 1, -e^2)
    s3, c3 = oracle.scaled_exp(np.array([0.0, -1.0, 1.0 + 1j * math.pi]))
    assert c3 == 1.0 and np.allclose(s3, [math.e, 1.0, -math.e ** 2], rtol=1e-15)
    # a vector of zeros stays zero
    s4, c4 = oracle.scaled_exp(oracle.to_goom(np.zeros(3)))
    assert np.all(s4 == 0) and np.isneginf(c4)


def test_signed_log_add(oracle):
    # the GOOM of a sum: against plain addition where everything is in range, and its algebra where not
    rng = np.random.default_rng(8)
    a = rng.standard_normal(2000) * np.exp(rng.uniform(-20, 20, 2000))
    b = rng.standard_normal(2000) * np.exp(rng.uniform(-20, 20, 2000))
    re, sg = oracle.log_add_exp(oracle.to_goom(a), oracle.to_goom(b))
    s = a + b
    # the logs of a and b are rounded to double: each carries a relative error of |log| * 2^-53 into the sum
    slack = (np.abs(np.log(np.abs(a))) * np.abs(a) + np.abs(np.log(np.abs(b))) * np.abs(b)) / np.abs(s) * 2.0 ** -52
    assert np.all(np.abs(re - np.log(np.abs(s))) <= 1e-15 * np.abs(re) + slack + 1e-15) and np.array_equal(sg, (s < 0).astype(np.uint8))
    re2, sg2 = oracle.log_add_exp(oracle.to_goom(b), oracle.to_goom(a))
    assert np.array_equal(re, re2) and np.array_equal(sg, sg2)  # commutative, bit for bit
    # far outside any float range: e^1000 + e^1000 = e^(1000 + ln 2); e^1000 - e^1000 = 0; x + 0 = x
    big = np.array([1000.0 + 0j, 1000.0 + 0j, 1000.0 + 1j * math.pi, -np.inf + 0j, -5000.0 + 0j])
    other = np.array([1000.0 + 0j, 1000.0 + 1j * math.pi, 999.0 + 0j, 3.0 + 1j * math.pi, -5000.0 + 1j * math.pi])
    re, sg = oracle.log_add_exp(big, other)
    assert abs(re[0] - (1000.0 + math.log(2.0))) < 1e-12 and sg[0] == 0
    assert np.isneginf(re[1]) and sg[1] == 0
    assert abs(re[2] - (1000.0 + math.log(1.0 - math.exp(-1.0)))) < 1e-12 and sg[2] == 1
    assert re[3] == 3.0 and sg[3] == 1
    assert np.isneginf(re[4])
    # it is the two-term case of the signed log-sum-exp that defines LMME: a 1 x 2 times 2 x 1 product
    for k in range(20):
        A = np.array([[oracle.to_goom(a[k:k + 1])[0], oracle.to_goom(b[k:k + 1])[0]]])
        ones = np.zeros((2, 1), dtype=np.complex128)
        r1, s1 = oracle.lmme(A, ones)
        assert abs(r1[0, 0] - re_k(oracle, a[k], b[k])) < 1e-13 and s1[0, 0] == (a[k] + b[k] < 0)


def re_k(oracle, x, y):
    return oracle.log_add_exp(oracle.to_goom(np.array([x])), oracle.to_goom(np.array([y])))[0][0]
