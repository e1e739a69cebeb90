"""Pins for the oracle's QR spectrum estimator and selectively reset recurrence (paper
Section 4.2.1, Section 5 and Appendix C).  No GPU."""
import math

import numpy as np
from scipy.special import digamma

import synthetic_inputs as si
from test_oracle_lmme_scan import goom_of


def real_of(re, sg):
    return np.where(sg == 1, -1.0, 1.0) * np.exp(re)


def test_qr_against_library(oracle):
    rng = np.random.default_rng(31)
    for d in (1, 2, 5, 32):
        a = rng.standard_normal((d, d))
        q, r = oracle.qr(a)
        assert np.allclose(q @ r, a, atol=1e-12) and np.allclose(q.T @ q, np.eye(d), atol=1e-12)
        assert np.all(np.diag(r) > 0) and np.allclose(np.tril(r, -1), 0)
        ql, rl = np.linalg.qr(a)
        s = np.sign(np.diag(rl))
        assert np.allclose(q, ql * s[None, :], atol=1e-10) and np.allclose(r, rl * s[:, None], atol=1e-10)


def test_spectrum_sums_to_mean_log_det(oracle):
    # sum of exponents = mean log|det J_t| / dt for any chain (each step's R has |det R| = |det J|)
    J, _ = si.lorenz96_jacobians(si.BASE_SEED + 7, 400, d=8, burn_in=500)
    lam = oracle.lyapunov_qr(J, 0.01)
    want = np.mean([np.linalg.slogdet(j.astype(np.float64))[1] for j in J]) / 0.01
    assert abs(lam.sum() - want) < 1e-8 * max(1, abs(want))
    assert np.all(np.diff(lam) < 0.5)  # roughly ordered
    # Lorenz-96: tr Df = -d, so the sum is -d + O(dt)
    assert abs(lam.sum() + 8) < 2.5  # log det(I + dt Df) = dt tr Df - dt^2 tr(Df^2) / 2 + ...


def test_gaussian_closed_form_spectrum(oracle):
    # products of i.i.d. N(0,1) d x d matrices: lambda_k = (ln 2 + psi((d - k + 1) / 2)) / 2, k = 1..d
    d, T = 4, 40000
    x = si.normal_chain(si.BASE_SEED + 8, T, d).astype(np.float64)
    lam = oracle.lyapunov_qr(x, 1.0)
    want = 0.5 * (math.log(2) + digamma((d - np.arange(1, d + 1) + 1) / 2))
    assert np.all(np.abs(lam - want) < 0.03), (lam, want)


def test_reset_never_equals_plain_scan(oracle):
    J = goom_of(np.random.default_rng(33).standard_normal((20, 5, 5)))
    X0 = goom_of(np.random.default_rng(34).standard_normal((5, 5)))
    re, sg, flag, growth = oracle.reset_scan(J, X0, check_every=4, policy=-1)
    re2, sg2 = oracle.scan(J, init=X0)
    assert np.array_equal(re, re2) and np.array_equal(sg, sg2) and flag.sum() == 0


def numpy_reset(x):
    """R of Section 4.2.1 (a) with numpy: unit columns, then the orthonormal factor, diag R > 0."""
    n = x / np.linalg.norm(x, axis=0, keepdims=True)
    q, r = np.linalg.qr(n)
    return q * np.sign(np.diag(r))[None, :]


def test_reset_worked_example_sequential(oracle):
    # Appendix C with one reset: the states after the reset are propagated from R(.)
    rng = np.random.default_rng(35)
    A = rng.standard_normal((3, 4, 4))
    X0 = rng.standard_normal((4, 4))
    re, sg, flag, _ = oracle.reset_scan(goom_of(A), goom_of(X0), check_every=2, policy=1)
    assert flag.tolist() == [0, 1, 0]
    x1 = A[0] @ X0
    x2 = numpy_reset(A[1] @ x1)
    x3 = A[2] @ x2
    for got, want in zip((real_of(re[0], sg[0]), real_of(re[1], sg[1]), real_of(re[2], sg[2])), (x1, x2, x3)):
        assert np.allclose(got, want, rtol=1e-9, atol=1e-12)


def test_reset_tuple_combine_reproduces_appendix_tables(oracle):
    # The literal (A*, B*) transformation of Section 5, eq. 28, applied in the order of the
    # two tables of Appendix C (right-to-left doubling scan over 4 elements).
    rng = np.random.default_rng(36)
    d = 3
    A1, A2, A3, X0 = (rng.standard_normal((d, d)) for _ in range(4))
    Z = np.zeros((d, d))
    R = lambda m: numpy_reset(m)

    def run(reset_second):
        e = [(X0.copy(), Z.copy()), (A1.copy(), Z.copy()), (A2.copy(), Z.copy()), (A3.copy(), Z.copy())]
        # parallel step 1: (1 <- 0) and (3 <- 2)
        p0, b0, c1, d1 = oracle.reset_combine_real(e[0][0], e[0][1], e[1][0], e[1][1], False, Z)
        p2, b2, c3, d3 = oracle.reset_combine_real(e[2][0], e[2][1], e[3][0], e[3][1], False, Z)
        e = [(p0, b0), (c1, d1), (p2, b2), (c3, d3)]
        sel = reset_second
        # parallel step 2: (2 <- 1) and (3 <- 1), with the reset decided on element 1
        rv = R(e[1][0]) if sel else Z
        p1, b1, c2, d2 = oracle.reset_combine_real(e[1][0], e[1][1], e[2][0], e[2][1], sel, rv)
        _, _, c3, d3 = oracle.reset_combine_real(e[1][0], e[1][1], e[3][0], e[3][1], sel, rv)
        return [e[0], (p1, b1), (c2, d2), (c3, d3)]

    plain = run(False)
    sums = [a + b for a, b in plain]
    assert all(np.all(b == 0) for _, b in plain)  # all bias slots stay zero
    for got, want in zip(sums, (X0, A1 @ X0, A2 @ A1 @ X0, A3 @ A2 @ A1 @ X0)):
        assert np.allclose(got, want, rtol=1e-12, atol=1e-13)
    withr = run(True)
    r1 = R(A1 @ X0)
    for (a, b), want in zip(withr[1:], (r1, A2 @ r1, A3 @ A2 @ r1)):
        assert np.all(a == 0) and np.allclose(b, want, rtol=1e-12, atol=1e-13)
    # the bias update uses A_curr before its own update: A_3 B_2 + B_3, not A_3 A_2 B_2 + B_3
    B2 = rng.standard_normal((d, d))
    B3 = rng.standard_normal((d, d))
    _, _, a, b = oracle.reset_combine_real(A2, B2, A3, B3, False, Z)
    assert np.allclose(a, A3 @ A2) and np.allclose(b, A3 @ B2 + B3)
    assert not np.allclose(b, A3 @ A2 @ B2 + B3)


def test_reset_scan_in_tree_order(oracle):
    # the whole scan in the paper's parallel order (Appendix C), literal tuples over reals
    rng = np.random.default_rng(37)
    d, T = 3, 11
    A = rng.standard_normal((T, d, d))
    X0 = rng.standard_normal((d, d))
    # S == 0: the plain recurrence, every bias slot stays zero
    sums, was = oracle.reset_scan_tree_real(X0, A, policy=-1)
    want = [X0]
    for t in range(T):
        want.append(A[t] @ want[-1])
    assert not was.any() and np.allclose(sums, np.stack(want), rtol=1e-12, atol=1e-13)
    # S == 1: every element is reset before the first parallel step, and a reset element ignores what precedes it
    sums, was = oracle.reset_scan_tree_real(X0, A, policy=1)
    assert was.all()
    for i, m in enumerate([X0] + list(A)):
        assert np.allclose(sums[i], numpy_reset(m), rtol=1e-10, atol=1e-12)
    # the appendix's second table: four elements, the compound A_1 X_0 selected (nearly parallel columns) and nothing
    # else: outputs X_0, R(A_1 X_0), A_2 R(A_1 X_0), A_3 A_2 R(A_1 X_0)
    def max_cos(m):
        n = m / np.linalg.norm(m, axis=0, keepdims=True)
        return np.abs((n.T @ n)[np.triu_indices(m.shape[0], 1)]).max()
    M = rng.standard_normal((d, d))
    M[:, 2] = M[:, 0] + 1e-6 * rng.standard_normal(d)  # the compound A_1 X_0: two nearly parallel columns
    A1 = M @ np.linalg.inv(X0)
    A2, A3 = rng.standard_normal((d, d)), rng.standard_normal((d, d))
    c = A1 @ X0
    assert max_cos(c) > 0.999999 and max(max_cos(m) for m in (X0, A1, A2, A3, A3 @ A2)) < 0.99
    sums, was = oracle.reset_scan_tree_real(X0, np.stack([A1, A2, A3]), policy=0, cos_threshold=0.999)
    r1 = numpy_reset(c)
    assert was.tolist() == [False, True, True, True]
    for got, want in zip(sums, (X0, r1, A2 @ r1, A3 @ A2 @ r1)):
        assert np.allclose(got, want, rtol=1e-9, atol=1e-11)


def test_reset_growth_equals_qr_spectrum(oracle):
    # triangular factors multiply, so the log-growth removed at resets (plus the final
    # factorisation) gives the same spectrum as QR at every step
    Jr, _ = si.lorenz96_jacobians(si.BASE_SEED + 9, 600, d=6, burn_in=300)
    lam = oracle.lyapunov_qr(Jr, 0.01)
    J = oracle.to_goom(Jr)
    for every, policy in ((50, 1), (64, 1), (7, 1), (600, -1)):
        _, _, flag, growth = oracle.reset_scan(J, None, check_every=every, policy=policy)
        assert np.allclose(growth / (600 * 0.01), lam, atol=1e-7), (every, policy)
    # colinearity-triggered policy resets less often than "always" but still often enough
    _, _, flag, growth = oracle.reset_scan(J, None, check_every=10, policy=0, cos_threshold=0.9)
    assert 0 < flag.sum() < 60
    assert np.allclose(growth / 6.0, lam, atol=1e-6)


def test_reset_states_are_orthonormal_after_reset(oracle):
    Jr, _ = si.lorenz96_jacobians(si.BASE_SEED + 10, 64, d=6, burn_in=100)
    re, sg, flag, _ = oracle.reset_scan(oracle.to_goom(Jr), None, check_every=16, policy=1)
    for t in np.nonzero(flag)[0]:
        q = real_of(re[t], sg[t])
        assert np.allclose(q.T @ q, np.eye(6), atol=1e-10)


# ------------------------------------------------- largest exponent (Section 4.2.2)

def test_lle_standard_is_first_exponent_of_qr_method(oracle):
    # with u_0 = e_1 the normalised vector iteration IS the first column of the QR iteration
    J, _ = si.lorenz96_jacobians(si.BASE_SEED + 9, 3000, d=8, burn_in=500)
    e1 = np.zeros(8)
    e1[0] = 1.0
    lle = oracle.lle_standard(J, e1, 0.01)
    assert abs(lle - oracle.lyapunov_qr(J, 0.01)[0]) < 1e-10
    # closed form for products of Gaussian matrices (d = 8): (ln 2 + psi(4)) / 2, any unit start
    T, d = 20000, 8
    G = si.normal_chain(si.BASE_SEED + 10, T, d)
    u0 = np.ones(d) / math.sqrt(d)
    want = 0.5 * (math.log(2.0) + digamma(d / 2))
    sigma = math.sqrt(0.25 * 0.2838 / T)  # var of log chi^2_8 / 4 per step, trigamma(4) = 0.2838
    assert abs(oracle.lle_standard(G, u0, 1.0) - want) < 5 * sigma + 1e-3


def test_lle_over_gooms_equals_standard_method(oracle):
    # without normalisation the sum telescopes to log|J_T ... J_1 u_0| / (dt T): LSE(2 x') / 2 over GOOMs
    T, d = 600, 8
    J, _ = si.lorenz96_jacobians(si.BASE_SEED + 11, T, d=d, burn_in=500)
    u0 = si.normal_f32(si.BASE_SEED + 11, 3, d).astype(np.float64)
    u0 /= np.linalg.norm(u0)
    want = oracle.lle_standard(J, u0, 0.01)
    Jz, uz = oracle.to_goom(J.astype(np.float64)), oracle.to_goom(u0)
    assert abs(oracle.lle_goom(Jz, uz, 0.01) - want) < 1e-9
    assert abs(oracle.lle_goom(Jz, uz, 0.01, scaled=True) - want) < 1e-9
    # far past double range: 3000 Gaussian 16 x 16 factors (log-norm about 4000)
    T, d = 3000, 16
    G = si.normal_chain(si.BASE_SEED + 12, T, d)
    u0 = np.ones(d) / math.sqrt(d)
    got = oracle.lle_goom(oracle.to_goom(G.astype(np.float64)), oracle.to_goom(u0), 1.0, scaled=True)
    assert abs(got - oracle.lle_standard(G, u0, 1.0)) < 1e-9 and got * T > 3500


# ------------------------------------- spectrum from input states (Section 4.2.1 (b)-(d))

def _input_states(oracle, Jz, L, policy):
    """S_0 = I, S_1 .. S_{T-1} from the selectively reset recurrence, in working form."""
    T, d, _ = Jz.shape
    re, sg, _, _ = oracle.reset_scan(Jz, None, check_every=L, policy=policy)
    eye_re = np.where(np.eye(d) > 0, 0.0, -np.inf)
    pre = np.concatenate([eye_re[None], re[:-1]])
    psg = np.concatenate([np.zeros((1, d, d), np.uint8), sg[:-1]])
    return pre, psg


def test_spectrum_from_states_equals_sequential_qr(oracle):
    # any basis of the same nested subspaces gives the same Q_{t-1}, hence the same R_t: the groups
    # (b)-(d) on selectively reset states reproduce the step-by-step method
    T, d = 300, 8
    J, _ = si.lorenz96_jacobians(si.BASE_SEED + 13, T, d=d, burn_in=500)
    Jz = oracle.to_goom(J.astype(np.float64))
    want = oracle.lyapunov_qr(J, 0.01)
    for L, policy in ((5, 1), (1, 1), (7, 0), (0, -1)):
        lam, steplog = oracle.lyapunov_from_states(_input_states(oracle, Jz, L, policy), J, 0.01)
        tol = 1e-8 if policy >= 0 else 1e-4  # never resetting: the states nearly collapse even in double
        assert np.abs(lam - want).max() < tol, (L, policy, np.abs(lam - want).max())
        # per step, sum_k log R_kk = log|det J_t|, whatever the basis
        dets = np.array([np.linalg.slogdet(j.astype(np.float64))[1] for j in J])
        assert np.abs(steplog.sum(axis=1) - dets).max() < (1e-9 if policy >= 0 else 1e-5)
    # using the OUTPUT state of each step instead of its input state is wrong, and shows
    re, sg, _, _ = oracle.reset_scan(Jz, None, check_every=5, policy=1)
    bad, _ = oracle.lyapunov_from_states((re, sg), J, 0.01)
    assert np.abs(bad - want).max() > 1e-3
