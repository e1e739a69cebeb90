"""ctypes front end of the CPU oracle (``goom_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``; never by the product package.  The module
only marshals numpy arrays into the C functions; all arithmetic is in the C file.

GOOM arrays cross this boundary in two forms:
  * complex64 / complex128 numpy arrays (real = log-magnitude, imag = 0 or pi), the
    storage format of the paper's implementation (Section 3);
  * the oracle's working form ``(re, sg)``: float64 log-magnitudes and uint8 signs
    (0 = non-negative, 1 = negative).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "goom_oracle.c")
_LIB = os.path.join(_HERE, "libgoom_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, libquadmath).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-Wall",
               _SRC, "-o", _LIB, "-lquadmath", "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_floor_f32.restype = C.c_float
        _lib.oracle_floor_f64.restype = C.c_double
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(C.c_int(n))


def floor_value(dtype) -> float:
    return float(lib().oracle_floor_f32() if np.dtype(dtype) == np.float32 else lib().oracle_floor_f64())


# ----------------------------------------------------------------------------- codecs

def to_goom(x: np.ndarray, zero_floor: bool = False) -> np.ndarray:
    """float32/float64 array -> complex64/complex128 GOOM array (Section 3.1)."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        y = np.empty(x.shape, dtype=np.complex64)
        lib().oracle_to_goom_f32(_p(x), _p(y), C.c_size_t(x.size), C.c_int(int(zero_floor)))
    elif x.dtype == np.float64:
        y = np.empty(x.shape, dtype=np.complex128)
        lib().oracle_to_goom_f64(_p(x), _p(y), C.c_size_t(x.size), C.c_int(int(zero_floor)))
    else:
        raise TypeError("to_goom: float32 or float64 expected")
    return y


def from_goom(z: np.ndarray) -> np.ndarray:
    """complex64/complex128 GOOM array -> float32/float64 array (Section 3.1)."""
    z = np.ascontiguousarray(z)
    if z.dtype == np.complex64:
        x = np.empty(z.shape, dtype=np.float32)
        lib().oracle_from_goom_f32(_p(z), _p(x), C.c_size_t(z.size))
    elif z.dtype == np.complex128:
        x = np.empty(z.shape, dtype=np.float64)
        lib().oracle_from_goom_f64(_p(z), _p(x), C.c_size_t(z.size))
    else:
        raise TypeError("from_goom: complex64 or complex128 expected")
    return x


def split(z: np.ndarray):
    """complex GOOM array -> (float64 log-magnitudes, uint8 signs)."""
    z = np.ascontiguousarray(z)
    re = np.empty(z.shape, dtype=np.float64)
    sg = np.empty(z.shape, dtype=np.uint8)
    if z.dtype == np.complex64:
        lib().oracle_split_c64(_p(z), _p(re), _p(sg), C.c_size_t(z.size))
    elif z.dtype == np.complex128:
        lib().oracle_split_c128(_p(z), _p(re), _p(sg), C.c_size_t(z.size))
    else:
        raise TypeError("split: complex64 or complex128 expected")
    return re, sg


def _as_working(z):
    """Accept a complex array or an (re, sg) pair."""
    if isinstance(z, tuple):
        return _c(z[0], np.float64), _c(z[1], np.uint8)
    return split(z)


# ------------------------------------------------------------------------------- LMME

def lmme(a, b, return_kappa: bool = False):
    """LMME over the last two axes; leading axes are a batch (Section 3.2, eq. 9)."""
    are, asg = _as_working(a)
    bre, bsg = _as_working(b)
    n, d = are.shape[-2:]
    d2, m = bre.shape[-2:]
    assert d == d2 and are.shape[:-2] == bre.shape[:-2]
    lead = are.shape[:-2]
    batch = int(np.prod(lead)) if lead else 1
    cre = np.empty(lead + (n, m), dtype=np.float64)
    csg = np.empty(lead + (n, m), dtype=np.uint8)
    kap = np.empty(lead + (n, m), dtype=np.float64) if return_kappa else None
    lib().oracle_lmme_batched(_p(are), _p(asg), _p(bre), _p(bsg), _p(cre), _p(csg), _p(kap),
                              C.c_long(batch), C.c_int(n), C.c_int(d), C.c_int(m))
    return (cre, csg, kap) if return_kappa else (cre, csg)


# ------------------------------------------------------------------------------- scan

def scan(mats, init=None, return_kappa: bool = False):
    """All prefix products P_t = M_t ... M_1 (init) of a [T, d, d] chain (Section 4.1)."""
    mre, msg = _as_working(mats)
    T, d, d2 = mre.shape
    assert d == d2
    if init is not None:
        ire, isg = _as_working(init)
        assert ire.shape[0] == d
        m = ire.shape[1]
    else:
        ire = isg = None
        m = d
    pre = np.empty((T, d, m), dtype=np.float64)
    psg = np.empty((T, d, m), dtype=np.uint8)
    kap = np.empty((T, d, m), dtype=np.float64) if return_kappa else None
    lib().oracle_scan(_p(mre), _p(msg), _p(ire), _p(isg), _p(pre), _p(psg), _p(kap),
                      C.c_long(T), C.c_int(d), C.c_int(m))
    return (pre, psg, kap) if return_kappa else (pre, psg)


class ScanStream:
    """Walk a long chain block by block, keeping only the running state.

    ``scaled=False`` uses the definitional log-sum-exp combine; ``scaled=True`` uses
    the scaled real-product oracle (see the C file), which is for long chains only.
    """

    def __init__(self, d: int, m: int | None = None, init=None, scaled: bool = False):
        self.d = d
        self.m = d if m is None else m
        self.scaled = scaled
        self.valid = 0
        if scaled:
            self.w = np.zeros((d, self.m), dtype=np.float64)
            self.e = np.zeros((self.m,), dtype=np.float64)
            if init is not None:
                ire, isg = _as_working(init)
                cmax = ire.max(axis=0)
                cmax = np.where(np.isfinite(cmax), cmax, 0.0)
                ex = np.ceil(cmax / np.log(2.0))
                self.w[...] = np.where(isg.astype(bool), -1.0, 1.0) * np.exp(ire - ex * np.log(2.0))
                self.e[...] = ex
                self.valid = 1
        else:
            self.re = np.full((d, self.m), -np.inf, dtype=np.float64)
            self.sg = np.zeros((d, self.m), dtype=np.uint8)
            if init is not None:
                ire, isg = _as_working(init)
                self.re[...] = ire
                self.sg[...] = isg
                self.valid = 1

    def advance(self, mats, sample_t=(), return_kappa: bool = False):
        """Consume a [Tb, d, d] block; return the prefixes at block-local steps sample_t."""
        mre, msg = _as_working(mats)
        Tb = mre.shape[0]
        st = np.ascontiguousarray(np.asarray(sample_t, dtype=np.int64))
        ns = st.size
        ore = np.empty((ns, self.d, self.m), dtype=np.float64)
        osg = np.empty((ns, self.d, self.m), dtype=np.uint8)
        kap = np.empty((ns, self.d, self.m), dtype=np.float64) if return_kappa else None
        if self.scaled:
            lib().oracle_scan_scaled_stream(_p(mre), _p(msg), _p(self.w), _p(self.e),
                                            C.c_int(self.valid), _p(st), C.c_long(ns), _p(ore),
                                            _p(osg), _p(kap), C.c_long(Tb), C.c_int(self.d),
                                            C.c_int(self.m))
        else:
            lib().oracle_scan_stream(_p(mre), _p(msg), _p(self.re), _p(self.sg),
                                     C.c_int(self.valid), _p(st), C.c_long(ns), _p(ore), _p(osg),
                                     _p(kap), C.c_long(Tb), C.c_int(self.d), C.c_int(self.m))
        self.valid = 1
        return (ore, osg, kap) if return_kappa else (ore, osg)


# ----------------------------------------------------------------------------- affine

def affine_scan(a, b, h0=None, return_kappa: bool = False):
    """h_t = A_t h_{t-1} + b_t over GOOMs (Section 4.3).  a: [..., T, d, d]; b: [..., T, d]."""
    are, asg = _as_working(a)
    bre, bsg = _as_working(b)
    T, d = bre.shape[-2:]
    lead = bre.shape[:-2]
    batch = int(np.prod(lead)) if lead else 1
    assert are.shape == lead + (T, d, d)
    if h0 is not None:
        h0re, h0sg = _as_working(h0)
        assert h0re.shape == lead + (d,)
    else:
        h0re = h0sg = None
    hre = np.empty(lead + (T, d), dtype=np.float64)
    hsg = np.empty(lead + (T, d), dtype=np.uint8)
    kap = np.empty(lead + (T, d), dtype=np.float64) if return_kappa else None
    lib().oracle_affine_scan_batched(_p(are), _p(asg), _p(bre), _p(bsg), _p(h0re), _p(h0sg),
                                     _p(hre), _p(hsg), _p(kap), C.c_long(batch), C.c_long(T),
                                     C.c_int(d))
    return (hre, hsg, kap) if return_kappa else (hre, hsg)


def affine_scan_backward(a, b, grad_h, h0=None, h=None):
    """Backward pass of the recurrence h_t = A_t h_{t-1} + b_t over GOOMs (Sections 3.1 and 4.3): given
    grad_h[..., t, i] = dL / d Re h'_t[i], returns (dL / d Re A', dL / d Re b', dL / d Re h0' or None, adjoints
    as (re, sg)).  a: [..., T, d, d]; b, grad_h: [..., T, d]; h: the forward states to use (default: computed here)."""
    are, asg = _as_working(a)
    bre, bsg = _as_working(b)
    T, d = bre.shape[-2:]
    lead = bre.shape[:-2]
    batch = int(np.prod(lead)) if lead else 1
    hre, hsg = affine_scan(a, b, h0) if h is None else _as_working(h)
    G = _c(grad_h, np.float64)
    assert G.shape == lead + (T, d)
    if h0 is not None:
        h0re, h0sg = _as_working(h0)
    gA = np.empty(lead + (T, d, d)); gb = np.empty(lead + (T, d))
    gh0 = np.empty(lead + (d,)) if h0 is not None else None
    lre = np.empty(lead + (T, d)); lsg = np.empty(lead + (T, d), dtype=np.uint8)
    v = lambda x: x.reshape((batch,) + x.shape[len(lead):])
    for q in range(batch):
        lib().oracle_affine_backward(_p(v(are)[q]), _p(v(asg)[q]), _p(v(bre)[q]), _p(v(bsg)[q]),
                                     _p(v(h0re)[q]) if h0 is not None else None, _p(v(h0sg)[q]) if h0 is not None else None,
                                     _p(v(hre)[q]), _p(v(hsg)[q]), _p(v(G)[q]), _p(v(gA)[q]), _p(v(gb)[q]),
                                     _p(v(gh0)[q]) if h0 is not None else None, _p(v(lre)[q]), _p(v(lsg)[q]),
                                     C.c_long(T), C.c_int(d))
    return gA, gb, gh0, (lre, lsg)


def affine_scan_backward_time_invariant(a, b, grad_h, h0=None, h=None):
    """Backward pass of h_t = A h_{t-1} + b_t with one matrix for all steps (the state-space layer of Section 4.3): the
    matrix enters every step, so its gradient is the sum over the steps of the time-varying recurrence's gradients.
    a: [..., d, d]; b, grad_h: [..., T, d].  Returns (dL / d Re A' [..., d, d], dL / d Re b', dL / d Re h0' or None)."""
    are, _ = _as_working(a)
    T = np.asarray(b).shape[-2]
    lead = are.shape[:-2]
    rep = np.ascontiguousarray(np.broadcast_to(np.asarray(a)[..., None, :, :], lead + (T,) + are.shape[-2:]))
    gA, gb, gh0, _ = affine_scan_backward(rep, b, grad_h, h0=h0, h=h)
    return np.asarray(gA.astype(np.longdouble).sum(axis=-3), dtype=np.float64), gb, gh0


def scan_backward(mats, grad_p, init=None, p=None):
    """Backward pass of the prefix scan P_t = M_t P_{t-1} over GOOMs (Sections 3.1, 4.1): given grad_p[t, i, k] =
    dL / d Re P'_t[i, k], returns (dL / d Re M' [T, d, d], dL / d Re init' [d, m] or None, adjoints as (re, sg)).
    mats: [T, d, d]; init: [d, m] or None (the identity); p: the forward states to use (default: computed here)."""
    mre, msg = _as_working(mats)
    T, d, _ = mre.shape
    if init is not None:
        ire, isg = _as_working(init)
        m = ire.shape[1]
    else:
        ire = isg = None
        m = d
    pre, psg = scan(mats, init) if p is None else _as_working(p)
    G = _c(grad_p, np.float64)
    assert G.shape == (T, d, m) and pre.shape == (T, d, m)
    gM = np.empty((T, d, d)); gI = np.empty((d, m)) if init is not None else None
    lre = np.empty((T, d, m)); lsg = np.empty((T, d, m), dtype=np.uint8)
    lib().oracle_scan_backward(_p(mre), _p(msg), _p(ire), _p(isg), _p(pre), _p(psg), _p(G), _p(gM), _p(gI), _p(lre), _p(lsg),
                               C.c_long(T), C.c_int(d), C.c_int(m))
    return gM, gI, (lre, lsg)


def lmme_backward(a, b, grad_c, c=None):
    """Backward pass of C' = LMME(A', B') (Sections 3.1, 3.2): given grad_c[..., i, k] = dL / d Re C'_ik, returns
    (dL / d Re A', dL / d Re B') as reals.  a: [..., n, d], b: [..., d, m]; c: the forward result to use (default:
    computed here by the definition)."""
    are, asg = _as_working(a)
    bre, bsg = _as_working(b)
    n, d = are.shape[-2:]
    m = bre.shape[-1]
    lead = are.shape[:-2]
    batch = int(np.prod(lead)) if lead else 1
    cre, csg = lmme(a, b) if c is None else _as_working(c)
    G = _c(grad_c, np.float64)
    assert G.shape == lead + (n, m) and bre.shape == lead + (d, m)
    gA = np.empty(lead + (n, d)); gB = np.empty(lead + (d, m))
    v = lambda x: x.reshape((batch,) + x.shape[len(lead):])
    for q in range(batch):
        lib().oracle_lmme_backward(_p(v(are)[q]), _p(v(asg)[q]), _p(v(bre)[q]), _p(v(bsg)[q]), _p(v(cre)[q]), _p(v(csg)[q]),
                                   _p(v(G)[q]), _p(v(gA)[q]), _p(v(gB)[q]), C.c_int(n), C.c_int(d), C.c_int(m))
    return gA, gB


def to_goom_backward(x, grad_re, eps: float):
    """Backward of float -> GOOM with the redefined derivatives of Section 3.1: grad_re * s(x) / (|x| + eps)."""
    x = _c(x, np.float64); g = _c(grad_re, np.float64)
    out = np.empty_like(x)
    lib().oracle_to_goom_backward(_p(x), _p(g), _p(out), C.c_double(eps), C.c_long(x.size))
    return out


def from_goom_backward(z, grad_x, eps: float):
    """Backward of GOOM -> float with the redefined derivative of Section 3.1: grad_x * (x + s(x) eps)."""
    re, sg = _as_working(z)
    g = _c(grad_x, np.float64)
    out = np.empty_like(re)
    lib().oracle_from_goom_backward(_p(re), _p(sg), _p(g), _p(out), C.c_double(eps), C.c_long(re.size))
    return out


# --------------------------------------------------------------------------- Lyapunov

def qr(a: np.ndarray):
    a = _c(a, np.float64)
    d = a.shape[0]
    q = np.empty((d, d), dtype=np.float64)
    r = np.empty((d, d), dtype=np.float64)
    lib().oracle_qr(_p(a), _p(q), _p(r), C.c_int(d))
    return q, r


def lyapunov_qr(J: np.ndarray, dt: float) -> np.ndarray:
    """Sequential-QR Lyapunov spectrum of a [T, d, d] real Jacobian chain (Section 4.2.1)."""
    J = _c(J, np.float64)
    T, d, _ = J.shape
    lam = np.empty((d,), dtype=np.float64)
    lib().oracle_lyapunov_qr(_p(J), C.c_long(T), C.c_int(d), C.c_double(dt), _p(lam))
    return lam


def reset_scan(jac, x0=None, check_every: int = 0, policy: int = 1, cos_threshold: float = 0.99):
    """Selectively reset chain X_t = J_t X_{t-1} (Section 5), states examined every
    ``check_every`` steps.  policy: 1 = reset at every examined step, 0 = reset when
    near-colinear, -1 = never.  Returns (re, sg, reset_flag, growth)."""
    jre, jsg = _as_working(jac)
    T, d, _ = jre.shape
    if x0 is not None:
        x0re, x0sg = _as_working(x0)
    else:
        x0re = x0sg = None
    sre = np.empty((T, d, d), dtype=np.float64)
    ssg = np.empty((T, d, d), dtype=np.uint8)
    flag = np.zeros((T,), dtype=np.uint8)
    growth = np.empty((d,), dtype=np.float64)
    lib().oracle_reset_scan(_p(jre), _p(jsg), _p(x0re), _p(x0sg), _p(sre), _p(ssg), _p(flag),
                            _p(growth), C.c_long(T), C.c_int(d), C.c_long(check_every),
                            C.c_int(policy), C.c_double(cos_threshold))
    return sre, ssg, flag, growth


def reset_combine_real(a_prev, b_prev, a_curr, b_curr, select_prev: bool, reset_value):
    """One application of the tuple transformation of Section 5 (eq. 28) on real matrices.
    Returns the updated (a_prev, b_prev, a_curr, b_curr)."""
    ap, bp, ac, bc = (np.array(v, dtype=np.float64, order="C") for v in (a_prev, b_prev, a_curr, b_curr))
    rv = _c(reset_value, np.float64)
    d = ap.shape[0]
    lib().oracle_reset_combine_real(_p(ap), _p(bp), _p(ac), _p(bc), C.c_int(int(select_prev)),
                                    _p(rv), C.c_int(d))
    return ap, bp, ac, bc


def reset_scan_tree_real(x0, a, policy: int = 0, cos_threshold: float = 0.99):
    """The selective-resetting scan of Section 5 in the order of the paper's parallel prefix scan (Appendix C), over
    plain real matrices with the literal tuple transformation (eq. 28).  Elements: (X_0, 0), (A_1, 0), ..., (A_T, 0).
    Parallel step k works on blocks of 2^k elements: every element of a block's upper half is updated from the last
    element of its lower half.  Before each parallel step every element whose transition slot is selected and whose
    bias slot is all zeros is reset in place (B* <- R(A*), A* <- 0), as in the appendix's second table.  S: any two
    columns with |cosine| above the threshold (policy 0), always (1), never (-1); R: unit columns, then the
    orthonormal factor of a QR with positive diagonal (Section 4.2.1 (a)).
    x0: [d, d]; a: [T, d, d] reals.  Returns (sums [T + 1, d, d] = A* + B* per element, was_reset [T + 1])."""
    x0 = _c(x0, np.float64)
    a = _c(a, np.float64)
    T, d, _ = a.shape
    n = T + 1
    As = [x0.copy()] + [a[t].copy() for t in range(T)]
    Bs = [np.zeros((d, d)) for _ in range(n)]
    zero = np.zeros((d, d))

    def selected(m):
        if policy == 1:
            return True
        if policy == -1:
            return False
        nrm = np.sqrt((m * m).sum(axis=0))
        if np.any(nrm == 0.0):
            return False
        g = (m / nrm).T @ (m / nrm)
        return bool(np.any(np.abs(g[np.triu_indices(d, 1)]) > cos_threshold))

    def reset_value(m):
        nrm = np.sqrt((m * m).sum(axis=0))
        q, _ = qr(m / np.where(nrm > 0, nrm, 1.0))
        return q

    half = 1
    while half < n:
        for i in range(n):  # selective reset, in place
            if not Bs[i].any() and As[i].any() and selected(As[i]):
                Bs[i] = reset_value(As[i])
                As[i] = zero.copy()
        for i in range(n):  # ordinary recurrence with bias: upper half of every block from the lower half's last element
            if i & half:
                j = (i & ~(half - 1) & ~half) + half - 1
                _, _, As[i], Bs[i] = reset_combine_real(As[j], Bs[j], As[i], Bs[i], False, zero)
        half *= 2
    sums = np.stack([x + y for x, y in zip(As, Bs)])
    was_reset = np.array([bool(y.any()) for y in Bs])
    return sums, was_reset


def lyapunov_from_states(prev_states, J: np.ndarray, dt: float):
    """Groups (b)-(d) of Section 4.2.1: prev_states = (re, sg) of S_0 .. S_{T-1} (working form),
    J the real Jacobians [T, d, d].  Returns (lambda [d], per-step log|diag R| [T, d])."""
    pre, psg = _as_working(prev_states)
    J = _c(J, np.float64)
    T, d, _ = J.shape
    assert pre.shape == (T, d, d)
    steplog = np.empty((T, d), dtype=np.float64)
    lam = np.empty((d,), dtype=np.float64)
    lib().oracle_lyapunov_from_states(_p(pre), _p(psg), _p(J), _p(steplog), _p(lam), C.c_long(T), C.c_int(d),
                                      C.c_double(dt))
    return lam, steplog


def lle_standard(J: np.ndarray, u0: np.ndarray, dt: float) -> float:
    """Largest Lyapunov exponent by the normalised vector iteration (Section 4.2.2, eqs. 21-22)."""
    J = _c(J, np.float64)
    u0 = _c(u0, np.float64)
    T, d, _ = J.shape
    f = lib().oracle_lle_standard
    f.restype = C.c_double
    return float(f(_p(J), _p(u0), C.c_long(T), C.c_int(d), C.c_double(dt)))


def lle_goom(jac, u0, dt: float, scaled: bool = False) -> float:
    """Largest Lyapunov exponent as LSE(2 * scan(J_T ... J_1 u_0)) / (2 dt T) (Section 4.2.2, eq. 24):
    jac [T, d, d] and u0 [d] are GOOMs; the product is walked by the scan oracle."""
    T, d, _ = np.asarray(jac).shape if not isinstance(jac, tuple) else jac[0].shape
    init = np.asarray(u0).reshape(d, 1)
    fre, _ = ScanStream(d, m=1, init=init, scaled=scaled).advance(jac, sample_t=[T - 1])
    f = lib().oracle_lle_from_final
    f.restype = C.c_double
    return float(f(_p(_c(fre.reshape(d), np.float64)), C.c_long(T), C.c_int(d), C.c_double(dt)))


def scaled_exp(z):
    """Scaled exponentiation of GOOM vectors over the last axis (Section 4.3, eq. 27):
    returns (scaled reals in [-e^2, e^2], c = max log-magnitude of every vector)."""
    re, sg = _as_working(z)
    d = re.shape[-1]
    n = int(np.prod(re.shape[:-1])) if re.ndim > 1 else 1
    scaled = np.empty(re.shape, dtype=np.float64)
    c = np.empty(re.shape[:-1], dtype=np.float64)
    lib().oracle_scaled_exp(_p(re), _p(sg), _p(scaled), _p(c), C.c_long(n), C.c_int(d))
    return scaled, c


def scaled_exp_backward(z, grad_scaled):
    """Backward of scaled_exp with the log-scaling constant detached (Section 4.3): gradients with respect to Re z."""
    re, sg = _as_working(z)
    d = re.shape[-1]
    n = int(np.prod(re.shape[:-1])) if re.ndim > 1 else 1
    g = _c(grad_scaled, np.float64)
    assert g.shape == re.shape
    out = np.empty(re.shape, dtype=np.float64)
    lib().oracle_scaled_exp_backward(_p(re), _p(sg), _p(g), _p(out), C.c_long(n), C.c_int(d))
    return out


def log_add_exp(x, y):
    """Elementwise signed log-add of two GOOM arrays: the GOOM of exp(x) + exp(y).  Returns (re, sg)."""
    xre, xsg = _as_working(x)
    yre, ysg = _as_working(y)
    assert xre.shape == yre.shape
    ore = np.empty(xre.shape, dtype=np.float64)
    osg = np.empty(xre.shape, dtype=np.uint8)
    lib().oracle_log_add_exp(_p(xre), _p(xsg), _p(yre), _p(ysg), _p(ore), _p(osg), C.c_long(xre.size))
    return ore, osg
