"""Pins of the oracle's backward passes (Section 3.1: redefined finite derivatives; Section 4.3: the recurrence)
against things other than the oracle itself: central finite differences of a long-double evaluation in the
value domain, closed forms, and the sum rule of log-domain gradients."""
import math

import numpy as np

import synthetic_inputs as si


def goom_of(x):
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(divide="ignore"):
        return np.log(np.abs(x)) + 1j * np.pi * (x < 0)


def loss_value_domain(A, b, h0, G):
    """L = sum_t sum_i G[t, i] log|h_t[i]| with h_t = A_t h_{t-1} + b_t evaluated in long double reals."""
    h = h0.astype(np.longdouble)
    L = np.longdouble(0)
    for t in range(A.shape[0]):
        h = (A[t].astype(np.longdouble) * h[None, :]).sum(axis=1) + b[t].astype(np.longdouble)
        L += (G[t].astype(np.longdouble) * np.log(np.abs(h))).sum()
    return L


def test_recurrence_backward_against_finite_differences(oracle):
    rng = np.random.default_rng(31)
    T, d = 9, 4
    A = rng.standard_normal((T, d, d)) * 0.8
    b = rng.standard_normal((T, d))
    h0 = rng.standard_normal(d)
    G = rng.standard_normal((T, d))
    gA, gb, gh0, _ = oracle.affine_scan_backward(goom_of(A), goom_of(b), G, h0=goom_of(h0))
    delta = 1e-5
    # d / d log|v| by scaling v with e^(+-delta)
    for (t, i, j) in [(0, 0, 0), (3, 1, 2), (8, 3, 3), (5, 2, 0), (1, 3, 1)]:
        Ap, Am = A.copy(), A.copy()
        Ap[t, i, j] *= math.exp(delta)
        Am[t, i, j] *= math.exp(-delta)
        fd = float((loss_value_domain(Ap, b, h0, G) - loss_value_domain(Am, b, h0, G)) / (2 * delta))
        assert abs(gA[t, i, j] - fd) < 1e-7 * max(1.0, abs(fd)), (t, i, j, gA[t, i, j], fd)
    for (t, i) in [(0, 1), (4, 0), (8, 2)]:
        bp, bm = b.copy(), b.copy()
        bp[t, i] *= math.exp(delta)
        bm[t, i] *= math.exp(-delta)
        fd = float((loss_value_domain(A, bp, h0, G) - loss_value_domain(A, bm, h0, G)) / (2 * delta))
        assert abs(gb[t, i] - fd) < 1e-7 * max(1.0, abs(fd))
    for j in range(d):
        hp, hm = h0.copy(), h0.copy()
        hp[j] *= math.exp(delta)
        hm[j] *= math.exp(-delta)
        fd = float((loss_value_domain(A, b, hp, G) - loss_value_domain(A, b, hm, G)) / (2 * delta))
        assert abs(gh0[j] - fd) < 1e-7 * max(1.0, abs(fd))


def test_recurrence_backward_sum_rule_and_closed_forms(oracle):
    # scaling all of A_t[i, :] and b_t[i] by e^s scales h_t[i] by e^s for the last step: the log-domain
    # gradients of a row add up to the adjoint times the state, which at the last step is G itself
    rng = np.random.default_rng(32)
    T, d = 40, 6
    A, b = si.recurrence_inputs(si.BASE_SEED + 80, 1, T, d)
    A, b = A[0].astype(np.float64) * 3.0, b[0].astype(np.float64)  # states far outside float range need not matter
    G = rng.standard_normal((T, d))
    gA, gb, gh0, (lre, lsg) = oracle.affine_scan_backward(goom_of(A), goom_of(b), G)
    assert gh0 is None
    assert np.allclose(gA[-1].sum(axis=1) + gb[-1], G[-1], rtol=1e-10, atol=1e-12)
    hre, hsg = oracle.affine_scan(goom_of(A), goom_of(b))
    lam_h = np.where(lsg ^ hsg, -1.0, 1.0) * np.exp(lre + hre)  # adjoint times state, step by step
    assert np.allclose(gA.sum(axis=2) + gb, lam_h, rtol=1e-9, atol=1e-12)
    # without an initial state the first matrix multiplies a zero vector: no gradient
    assert np.all(gA[0] == 0.0)
    # scalar recurrence with a = 0: h_t = b_t, so dL / d log|b_t| = G_t
    gA1, gb1, _, _ = oracle.affine_scan_backward(goom_of(np.zeros((5, 1, 1))), goom_of(np.array([[2.0], [-3.0], [0.5], [4.0], [-1.0]])),
                                                 np.array([[1.0], [2.0], [3.0], [4.0], [5.0]]))
    assert np.allclose(gb1[:, 0], [1, 2, 3, 4, 5]) and np.all(gA1 == 0)
    # scalar, b = 0, h0 = 1: h_t = a^t, L = sum_t G_t t log a: dL / d log a_s = sum_{t >= s} G_t
    a = np.full((4, 1, 1), 1.7)
    Gs = np.array([[1.0], [10.0], [100.0], [1000.0]])
    gA2, _, gh02, _ = oracle.affine_scan_backward(goom_of(a), goom_of(np.zeros((4, 1))), Gs, h0=goom_of(np.array([1.0])))
    assert np.allclose(gA2[:, 0, 0], [1111.0, 1110.0, 1100.0, 1000.0]) and np.allclose(gh02, [1111.0])


def test_recurrence_backward_far_outside_float_range(oracle):
    # states of magnitude e^(+-thousands): the adjoints are as small as the states are large, the gradients stay O(G)
    rng = np.random.default_rng(33)
    T, d = 300, 5
    A = goom_of(rng.standard_normal((T, d, d))) + 30.0  # every entry times e^30
    b = goom_of(rng.standard_normal((T, d)))
    G = rng.standard_normal((T, d))
    gA, gb, _, (lre, _) = oracle.affine_scan_backward(A, b, G)
    hre, _ = oracle.affine_scan(A, b)
    assert hre.max() > 8000 and lre.min() < -8000
    assert np.isfinite(gA).all() and np.abs(gA).max() < 1e6
    assert np.allclose(gA[-1].sum(axis=1) + gb[-1], G[-1], rtol=1e-9, atol=1e-12)
    # a common shift of all log-magnitudes of A changes no gradient of A (only relative sizes enter)
    gA2, _, _, _ = oracle.affine_scan_backward(A + 5.0, b + 5.0 * (np.arange(T)[:, None] + 1), G)
    assert np.allclose(gA2, gA, rtol=1e-6, atol=1e-9)  # (log-magnitudes near 1e4 carry 2e-12 each into the exponentials)


def test_codec_backward_redefined_derivatives(oracle):
    # Section 3.1: d abs(x)/dx := +-1 (never 0, +1 at zero); d log(u)/du := 1/(u + eps); d exp(x')/dx' := exp(x') +- eps
    eps = 2.0 ** -20
    x = np.array([2.0, -2.0, 0.0, -0.0, 1e-30, -1e-30, 5.0])
    g = np.array([1.0, 1.0, 3.0, 3.0, 1.0, 1.0, -2.0])
    gx = oracle.to_goom_backward(x, g, eps)
    assert np.allclose(gx, [1 / (2 + eps), -1 / (2 + eps), 3 / eps, 3 / eps, 1 / (1e-30 + eps), -1 / (1e-30 + eps), -2 / (5 + eps)], rtol=1e-15)
    assert np.all(np.isfinite(gx)) and np.all(gx != 0)
    # away from zero it is the ordinary derivative of log|x|: central differences
    for v in (0.3, -7.0, 123.0):
        fd = (math.log(abs(v * (1 + 1e-6))) - math.log(abs(v * (1 - 1e-6)))) / (2e-6 * v)
        assert abs(oracle.to_goom_backward(np.array([v]), np.array([1.0]), 0.0)[0] - fd) < 1e-8 * abs(fd)
    z = np.array([math.log(3.0), math.log(3.0) + 1j * math.pi, -np.inf, -800.0 + 1j * math.pi, 1.5])
    gz = oracle.from_goom_backward(z, np.array([1.0, 1.0, 2.0, 2.0, -1.0]), eps)
    want = [3 + eps, -3 - eps, 2 * eps, -2 * eps, -(math.exp(1.5) + eps)]
    assert np.allclose(gz, want, rtol=1e-14) and np.all(gz != 0)
    # and the ordinary derivative of +-exp(re) with respect to re when eps = 0
    assert np.allclose(oracle.from_goom_backward(z[[0, 1, 4]], np.ones(3), 0.0), [3.0, -3.0, math.exp(1.5)], rtol=1e-15)


def lmme_loss_value_domain(A, B, G):
    """L = sum_ik G[i, k] log|(A B)[i, k]| in long double reals."""
    Cm = (A.astype(np.longdouble)[:, :, None] * B.astype(np.longdouble)[None, :, :]).sum(axis=1)
    return (G.astype(np.longdouble) * np.log(np.abs(Cm))).sum()


def test_lmme_backward_against_finite_differences(oracle):
    rng = np.random.default_rng(41)
    n, d, m = 5, 7, 4
    A = rng.standard_normal((n, d)) * np.exp(rng.uniform(-3, 3, (n, d)))
    B = rng.standard_normal((d, m)) * np.exp(rng.uniform(-3, 3, (d, m)))
    G = rng.standard_normal((n, m))
    gA, gB = oracle.lmme_backward(goom_of(A), goom_of(B), G)
    delta = 1e-5
    for (i, j) in [(0, 0), (4, 6), (2, 3), (1, 5), (3, 1)]:
        Ap, Am = A.copy(), A.copy()
        Ap[i, j] *= math.exp(delta)
        Am[i, j] *= math.exp(-delta)
        fd = float((lmme_loss_value_domain(Ap, B, G) - lmme_loss_value_domain(Am, B, G)) / (2 * delta))
        assert abs(gA[i, j] - fd) < 1e-7 * max(1.0, abs(fd)), (i, j, gA[i, j], fd)
    for (j, k) in [(0, 0), (6, 3), (3, 2), (5, 1), (1, 0)]:
        Bp, Bm = B.copy(), B.copy()
        Bp[j, k] *= math.exp(delta)
        Bm[j, k] *= math.exp(-delta)
        fd = float((lmme_loss_value_domain(A, Bp, G) - lmme_loss_value_domain(A, Bm, G)) / (2 * delta))
        assert abs(gB[j, k] - fd) < 1e-7 * max(1.0, abs(fd)), (j, k, gB[j, k], fd)
    # a transposed operand would pass the square case only: the shapes here are all different


def test_lmme_backward_sum_rules_and_special_cases(oracle):
    rng = np.random.default_rng(42)
    n, d, m = 6, 9, 8
    A = goom_of(rng.standard_normal((n, d))) + rng.uniform(-4000, 4000, (n, 1))  # rows far outside float range
    B = goom_of(rng.standard_normal((d, m))) + rng.uniform(-4000, 4000, (1, m))
    G = rng.standard_normal((n, m))
    gA, gB = oracle.lmme_backward(A, B, G)
    # scaling row i of A by e^s adds s to row i of log|C|: the gradients of a row of A' add up to those of the row of C';
    # likewise for the columns of B'
    assert np.allclose(gA.sum(axis=1), G.sum(axis=1), rtol=1e-9, atol=1e-11)
    assert np.allclose(gB.sum(axis=0), G.sum(axis=0), rtol=1e-9, atol=1e-11)
    # scaling column j of A by e^s and row j of B by e^-s changes nothing
    assert np.allclose(gA.sum(axis=0), gB.sum(axis=1), rtol=1e-9, atol=1e-11)
    # the row and column shifts themselves change no gradient
    gA0, gB0 = oracle.lmme_backward(goom_of(np.exp(A.real - A.real.max(axis=1, keepdims=True)) * np.cos(A.imag)),
                                    goom_of(np.exp(B.real - B.real.max(axis=0, keepdims=True)) * np.cos(B.imag)), G)
    assert np.allclose(gA, gA0, rtol=1e-8, atol=1e-10) and np.allclose(gB, gB0, rtol=1e-8, atol=1e-10)
    # inner dimension 1: C_ik = a_i b_k, so every term is G_ik itself
    a1, b1 = goom_of(np.array([[2.0], [-3.0]])), goom_of(np.array([[0.5, -4.0, 7.0]]))
    G1 = np.array([[1.0, 2.0, 3.0], [10.0, 20.0, 30.0]])
    gA1, gB1 = oracle.lmme_backward(a1, b1, G1)
    assert np.allclose(gA1[:, 0], [6.0, 60.0]) and np.allclose(gB1[0], [11.0, 22.0, 33.0])
    # identity right operand: C = A, the gradient goes straight through; that of B' is G_ik A_ij / A_ik summed over i
    Av = rng.standard_normal((3, 3)) + 2.0
    gA2, gB2 = oracle.lmme_backward(goom_of(Av), goom_of(np.eye(3)), np.ones((3, 3)))
    assert np.allclose(gA2, np.ones((3, 3)))
    assert np.allclose(gB2, np.eye(3) * 3.0)  # off-diagonal entries of B are zero: log-domain gradient A_ij B_jk / C_ik = 0
    # zero entries of the operands and zero gradients pass nothing; an exactly zero output passes nothing
    Az = np.array([[1.0, 0.0], [1.0, -1.0]])
    Bz = np.array([[1.0, 2.0], [1.0, 3.0]])
    gA3, gB3 = oracle.lmme_backward(goom_of(Az), goom_of(Bz), np.array([[1.0, 1.0], [5.0, 1.0]]))  # C[1, 0] = 0 exactly
    assert gA3[0, 1] == 0.0 and np.isfinite(gA3).all() and np.isfinite(gB3).all()
    assert np.allclose(gA3[0], [2.0, 0.0])
    assert np.allclose(gA3[1], [2.0 / -1.0, -3.0 / -1.0])  # only C[1, 1] = 2 - 3 = -1 contributes
    # batched leading axes
    Ab = goom_of(rng.standard_normal((2, 3, 4, 5)))
    Bb = goom_of(rng.standard_normal((2, 3, 5, 2)))
    Gb = rng.standard_normal((2, 3, 4, 2))
    gAb, gBb = oracle.lmme_backward(Ab, Bb, Gb)
    gAq, gBq = oracle.lmme_backward(Ab[1, 2], Bb[1, 2], Gb[1, 2])
    assert np.array_equal(gAb[1, 2], gAq) and np.array_equal(gBb[1, 2], gBq)


def scan_loss_value_domain(M, S0, G):
    """L = sum_t sum_ik G[t, i, k] log|P_t[i, k]| with P_t = M_t P_{t-1}, P_{-1} = S0 (the identity if None), in long double."""
    P = np.eye(M.shape[1], dtype=np.longdouble) if S0 is None else S0.astype(np.longdouble)
    L = np.longdouble(0)
    for t in range(M.shape[0]):
        P = (M[t].astype(np.longdouble)[:, :, None] * P[None, :, :]).sum(axis=1)
        L += (G[t].astype(np.longdouble) * np.log(np.abs(P))).sum()
    return L


def test_scan_backward_against_finite_differences(oracle):
    rng = np.random.default_rng(51)
    T, d, m = 7, 4, 3
    M = rng.standard_normal((T, d, d)) * 0.9
    S0 = rng.standard_normal((d, m))
    G = rng.standard_normal((T, d, m))
    delta = 1e-5
    for init in (S0, None):
        Gi = G if init is not None else rng.standard_normal((T, d, d))
        gM, gI, _ = oracle.scan_backward(goom_of(M), Gi, init=None if init is None else goom_of(init))
        for (t, i, j) in [(0, 0, 0), (0, 2, 3), (3, 1, 2), (6, 3, 3), (5, 2, 0), (1, 3, 1), (6, 0, 2)]:
            Mp, Mm = M.copy(), M.copy()
            Mp[t, i, j] *= math.exp(delta)
            Mm[t, i, j] *= math.exp(-delta)
            fd = float((scan_loss_value_domain(Mp, init, Gi) - scan_loss_value_domain(Mm, init, Gi)) / (2 * delta))
            assert abs(gM[t, i, j] - fd) < 1e-7 * max(1.0, abs(fd)), (t, i, j, gM[t, i, j], fd)
        if init is None:
            assert gI is None
            continue
        for (j, k) in [(0, 0), (3, 2), (1, 1), (2, 0)]:
            Sp, Sm = S0.copy(), S0.copy()
            Sp[j, k] *= math.exp(delta)
            Sm[j, k] *= math.exp(-delta)
            fd = float((scan_loss_value_domain(M, Sp, G) - scan_loss_value_domain(M, Sm, G)) / (2 * delta))
            assert abs(gI[j, k] - fd) < 1e-7 * max(1.0, abs(fd)), (j, k, gI[j, k], fd)


def test_scan_backward_sum_rules_and_special_cases(oracle):
    rng = np.random.default_rng(52)
    T, d, m = 60, 5, 3
    M = goom_of(rng.standard_normal((T, d, d))) + 25.0   # every entry times e^25: states of magnitude e^(25 t)
    S0 = goom_of(rng.standard_normal((d, m)))
    G = rng.standard_normal((T, d, m))
    gM, gI, (lre, lsg) = oracle.scan_backward(M, G, init=S0)
    pre, psg = oracle.scan(M, S0)
    assert pre.max() > 1400 and lre.min() < -1400 and np.isfinite(gM).all() and np.abs(gM).max() < 1e7
    # scaling row i of M_t by e^s scales row i of P_t and, through the later factors, every later state:
    # sum_j gM_t[i, j] = sum_k (adjoint times state)_t[i, k]; at the last step that is sum_k G[i, k]
    lam_p = np.where(lsg ^ psg, -1.0, 1.0) * np.exp(lre + pre)
    assert np.allclose(gM.sum(axis=2), lam_p.sum(axis=2), rtol=1e-8, atol=1e-10)
    assert np.allclose(gM[-1].sum(axis=1), G[-1].sum(axis=1), rtol=1e-9, atol=1e-11)
    # scaling the whole of M_t by e^s adds s to every log-magnitude of P_u, u >= t: the gradients of M_t add up to sum_{u >= t} sum G_u
    tail = np.cumsum(G.sum(axis=(1, 2))[::-1])[::-1]
    assert np.allclose(gM.sum(axis=(1, 2)), tail, rtol=1e-7, atol=1e-9)
    # scaling column k of S0 scales column k of every state; scaling row j of S0 by e^s and column j of M_0 by e^-s changes nothing
    assert np.allclose(gI.sum(axis=0), G.sum(axis=(0, 1)), rtol=1e-7, atol=1e-9)
    assert np.allclose(gI.sum(axis=1), gM[0].sum(axis=0), rtol=1e-7, atol=1e-9)
    # between neighbouring factors: scaling column j of M_{t+1} by e^-s and row j of M_t by e^s changes only row j of P_t
    assert np.allclose(gM[1:].sum(axis=1), gM[:-1].sum(axis=2) - G[:-1].sum(axis=2), rtol=1e-7, atol=1e-9)
    # a common shift of all log-magnitudes changes no gradient
    gM2, gI2, _ = oracle.scan_backward(M + 3.0, G, init=S0 - 7.0)
    assert np.allclose(gM2, gM, rtol=1e-7, atol=1e-9) and np.allclose(gI2, gI, rtol=1e-7, atol=1e-9)
    # one step is an LMME: the same gradients as its backward pass
    gM1, gI1, _ = oracle.scan_backward(M[:1], G[:1], init=S0)
    gA, gB = oracle.lmme_backward(M[0], S0, G[0])
    assert np.allclose(gM1[0], gA, rtol=1e-12) and np.allclose(gI1, gB, rtol=1e-12)
    # scalars, no initial state: P_t = a_0 ... a_t, dL / d log a_s = sum_{t >= s} G_t
    a = goom_of(np.array([1.5, -0.5, 2.0, -3.0]).reshape(4, 1, 1))
    Gs = np.array([1.0, 10.0, 100.0, 1000.0]).reshape(4, 1, 1)
    g1, none, _ = oracle.scan_backward(a, Gs)
    assert none is None and np.allclose(g1[:, 0, 0], [1111.0, 1110.0, 1100.0, 1000.0])
    # diagonal factors, no initial state: every state is diagonal, off-diagonal entries are zero and pass nothing
    D = np.zeros((3, 2, 2)); D[:, 0, 0] = [2.0, 3.0, 4.0]; D[:, 1, 1] = [-1.0, 5.0, 0.5]
    gD, _, _ = oracle.scan_backward(goom_of(D), np.ones((3, 2, 2)))
    assert np.allclose(gD[:, 0, 0], [3, 2, 1]) and np.allclose(gD[:, 1, 1], [3, 2, 1]) and np.all(gD[:, 0, 1] == 0) and np.all(gD[:, 1, 0] == 0)


def test_time_invariant_recurrence_backward(oracle):
    # one matrix for all steps: finite differences move the matrix entry at every step at once
    rng = np.random.default_rng(61)
    T, d = 11, 3
    A = rng.standard_normal((d, d)) * 0.9
    b = rng.standard_normal((T, d))
    h0 = rng.standard_normal(d)
    G = rng.standard_normal((T, d))
    gA, gb, gh0 = oracle.affine_scan_backward_time_invariant(goom_of(A), goom_of(b), G, h0=goom_of(h0))
    rep = lambda M: np.broadcast_to(M, (T, d, d))
    delta = 1e-5
    for i in range(d):
        for j in range(d):
            Ap, Am = A.copy(), A.copy()
            Ap[i, j] *= math.exp(delta)
            Am[i, j] *= math.exp(-delta)
            fd = float((loss_value_domain(rep(Ap), b, h0, G) - loss_value_domain(rep(Am), b, h0, G)) / (2 * delta))
            assert abs(gA[i, j] - fd) < 1e-6 * max(1.0, abs(fd)), (i, j, gA[i, j], fd)  # (a state near zero: the difference quotient's own error is 1e-7)
    for (t, i) in [(0, 1), (5, 0), (10, 2)]:
        bp, bm = b.copy(), b.copy()
        bp[t, i] *= math.exp(delta)
        bm[t, i] *= math.exp(-delta)
        fd = float((loss_value_domain(rep(A), bp, h0, G) - loss_value_domain(rep(A), bm, h0, G)) / (2 * delta))
        assert abs(gb[t, i] - fd) < 1e-7 * max(1.0, abs(fd))
    # scalar, no bias, h0 = 1: h_t = a^(t + 1), L = sum_t G_t (t + 1) log a
    Gs = np.array([[1.0], [10.0], [100.0]])
    g1, _, g01 = oracle.affine_scan_backward_time_invariant(goom_of(np.array([[1.3]])), goom_of(np.zeros((3, 1))), Gs, h0=goom_of(np.array([1.0])))
    assert np.allclose(g1, [[321.0]]) and np.allclose(g01, [111.0])
    # batched leading axes, and the same bias and state gradients as the time-varying pass on the repeated matrix
    Ab = goom_of(rng.standard_normal((2, d, d)))
    bb = goom_of(rng.standard_normal((2, T, d)))
    Gb = rng.standard_normal((2, T, d))
    gAb, gbb, none = oracle.affine_scan_backward_time_invariant(Ab, bb, Gb)
    gA1, gb1, _ = oracle.affine_scan_backward_time_invariant(Ab[1], bb[1], Gb[1])
    assert none is None and np.array_equal(gAb[1], gA1) and np.array_equal(gbb[1], gb1)
    full, gbf, _, _ = oracle.affine_scan_backward(np.broadcast_to(Ab[:, None], (2, T, d, d)).copy(), bb, Gb)
    assert np.allclose(gAb, full.sum(axis=1), rtol=1e-13) and np.array_equal(gbb, gbf)


def test_scaled_exp_backward_constant_detached(oracle):
    # Section 4.3: c = max Re z takes no gradient.  With c held at its value, scaled_i = +-exp(re_i - c + 2) and the derivative
    # with respect to re_i is scaled_i itself, also for the entry that sets c (were c differentiated, that entry's would be 0)
    rng = np.random.default_rng(71)
    z = goom_of(rng.standard_normal((3, 6)) * np.exp(rng.uniform(-5, 5, (3, 6)))) + np.array([[900.0], [-4000.0], [0.0]])
    g = rng.standard_normal((3, 6))
    got = oracle.scaled_exp_backward(z, g)
    scaled, c = oracle.scaled_exp(z)
    assert np.allclose(got, g * scaled, rtol=1e-15)
    top = np.argmax(z.real, axis=1)
    assert np.allclose(got[np.arange(3), top], g[np.arange(3), top] * np.where(z.imag[np.arange(3), top] != 0, -1, 1) * math.exp(2.0), rtol=1e-14)
    delta = 1e-6
    for (v, i) in [(0, 0), (1, 3), (2, 5), (0, int(top[0]))]:
        f = lambda r: math.exp(r - c[v] + 2.0) * (-1.0 if z.imag[v, i] != 0 else 1.0)  # c fixed
        fd = g[v, i] * (f(z.real[v, i] + delta) - f(z.real[v, i] - delta)) / (2 * delta)
        assert abs(got[v, i] - fd) < 1e-8 * max(1.0, abs(fd))
    # a vector of zeros passes nothing
    assert np.all(oracle.scaled_exp_backward(np.full((1, 4), -np.inf + 0j), np.ones((1, 4))) == 0)
