"""ctypes binding over libgoom's C ABI (``include/goom.h``), same names as the C calls.

Marshalling only: every step of the computation runs in the HIP kernels.  PyTorch is
used for device memory and streams.  Tensors must be contiguous CUDA (ROCm) tensors on
the context's device; complex64 / complex128 tensors carry GOOMs (real = log-magnitude,
imag = 0 or pi).
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgoom.so")
_lib = None

C64, C128 = 0, 1
ZERO_NEG_INF, ZERO_FLOOR = 0, 1
LMME_FAST, LMME_EXACT = 0, 1
RESET_ALWAYS, RESET_COLINEAR, RESET_NEVER = 1, 0, -1
AFFINE_TIME_INVARIANT = 1

EXPORTS = [
    "goom_version", "goom_create", "goom_destroy", "goom_set_stream", "goom_last_error",
    "goom_status_name", "goom_probe_bandwidth", "goom_probe_matrix_unit", "goom_profile_enable", "goom_profile_count", "goom_profile_get", "goom_to_goom", "goom_from_goom", "goom_lmme", "goom_lmme_workspace_bytes",
    "goom_scan", "goom_scan_workspace_bytes", "goom_scan_static", "goom_reduce", "goom_reduce_workspace_bytes",
    "goom_scan_real", "goom_scan_real_workspace_bytes", "goom_reduce_real", "goom_reduce_real_workspace_bytes",
    "goom_scan_reset", "goom_scan_reset_workspace_bytes", "goom_scan_reset_tree", "goom_scan_reset_tree_workspace_bytes", "goom_lyapunov_spectrum",
    "goom_lyapunov_spectrum_per_step", "goom_lyapunov_spectrum_per_step_workspace_bytes",
    "goom_largest_lyapunov", "goom_largest_lyapunov_workspace_bytes",
    "goom_affine_scan", "goom_affine_scan_workspace_bytes", "goom_affine_scan_scaled",
    "goom_affine_scan_scaled_workspace_bytes", "goom_scaled_exp", "goom_log_add_exp",
    "goom_count_nonfinite", "goom_to_goom_backward", "goom_from_goom_backward", "goom_affine_scan_backward", "goom_affine_scan_backward_workspace_bytes",
    "goom_lmme_backward", "goom_lmme_backward_workspace_bytes", "goom_scan_backward", "goom_scan_backward_workspace_bytes", "goom_scaled_exp_backward",
]


class GoomError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{status_name(status)}: {message}")
        self.status = status


class ScanOpts(C.Structure):
    _fields_ = [("chunk_len", C.c_int64), ("flags", C.c_uint32)]


class ResetOpts(C.Structure):
    _fields_ = [("chunk_len", C.c_int64), ("policy", C.c_int32), ("cos_threshold", C.c_float)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libgoom.so.  It must have been built (``python -m paper_2510_03426_amd.build`` or
    ``__graft_entry__.build()``); there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise GoomErrorNoLib()
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, u32, sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint32, C.c_size_t
    lib.goom_version.restype = i32
    lib.goom_create.argtypes = [C.POINTER(vp), i32, vp]
    lib.goom_destroy.argtypes = [vp]
    lib.goom_set_stream.argtypes = [vp, vp]
    lib.goom_last_error.argtypes = [vp]
    lib.goom_last_error.restype = C.c_char_p
    lib.goom_status_name.argtypes = [i32]
    lib.goom_status_name.restype = C.c_char_p
    lib.goom_profile_enable.argtypes = [vp, i32]
    lib.goom_profile_count.argtypes = [vp]
    lib.goom_profile_get.argtypes = [vp, i32, C.POINTER(C.c_char_p), C.POINTER(C.c_float)]
    lib.goom_to_goom.argtypes = [vp, vp, vp, sz, i32, u32]
    lib.goom_from_goom.argtypes = [vp, vp, vp, sz, i32]
    lib.goom_lmme.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, i32, u32, vp, sz]
    lib.goom_lmme_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, u32]
    lib.goom_lmme_workspace_bytes.restype = sz
    po = C.POINTER(ScanOpts)
    lib.goom_scan.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, i32, po, vp, sz]
    lib.goom_scan_workspace_bytes.argtypes = [i64, i32, i32, i64, i32, po]
    lib.goom_scan_workspace_bytes.restype = sz
    lib.goom_scan_static.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, i32, po]
    lib.goom_reduce.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, i32, po, vp, sz]
    lib.goom_reduce_workspace_bytes.argtypes = [i64, i32, i32, i64, i32, po]
    lib.goom_reduce_workspace_bytes.restype = sz
    lib.goom_scan_real.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, i32, po, vp, sz]
    lib.goom_scan_real_workspace_bytes.argtypes = [i64, i32, i32, i64, i32, po]
    lib.goom_scan_real_workspace_bytes.restype = sz
    lib.goom_reduce_real.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, i32, po, vp, sz]
    lib.goom_reduce_real_workspace_bytes.argtypes = [i64, i32, i32, i64, i32, po]
    lib.goom_reduce_real_workspace_bytes.restype = sz
    pr = C.POINTER(ResetOpts)
    lib.goom_scan_reset.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i64, i32, pr, vp, sz]
    lib.goom_scan_reset_workspace_bytes.argtypes = [i64, i32, i64, i32, pr]
    lib.goom_scan_reset_workspace_bytes.restype = sz
    lib.goom_scan_reset_tree.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32, pr, vp, sz]
    lib.goom_scan_reset_tree_workspace_bytes.argtypes = [i64, i32, i64, i32]
    lib.goom_scan_reset_tree_workspace_bytes.restype = sz
    lib.goom_lyapunov_spectrum.argtypes = [vp, vp, vp, vp, vp, i64, i32, C.c_double, i64, i32, pr, vp, sz]
    lib.goom_lyapunov_spectrum_per_step.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, C.c_double, i64, i32, pr, vp, sz]
    lib.goom_lyapunov_spectrum_per_step_workspace_bytes.argtypes = [i64, i32, i64, i32, pr, i32, i32]
    lib.goom_lyapunov_spectrum_per_step_workspace_bytes.restype = sz
    lib.goom_largest_lyapunov.argtypes = [vp, vp, vp, vp, i64, i32, C.c_double, i64, i32, po, vp, sz]
    lib.goom_largest_lyapunov_workspace_bytes.argtypes = [i64, i32, i64, i32, po]
    lib.goom_largest_lyapunov_workspace_bytes.restype = sz
    lib.goom_scaled_exp.argtypes = [vp, vp, vp, vp, sz, i32, i32]
    lib.goom_log_add_exp.argtypes = [vp, vp, vp, vp, sz, i32]
    lib.goom_affine_scan.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32, po, vp, sz]
    lib.goom_affine_scan_workspace_bytes.argtypes = [i64, i32, i64, i32, po]
    lib.goom_affine_scan_workspace_bytes.restype = sz
    lib.goom_probe_bandwidth.argtypes = [vp, vp, vp, sz, i32]
    lib.goom_probe_matrix_unit.argtypes = [vp, vp, i64, i32]
    lib.goom_affine_scan_scaled.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i64, i32, po, vp, sz]
    lib.goom_affine_scan_scaled_workspace_bytes.argtypes = [i64, i32, i64, i32, po]
    lib.goom_affine_scan_scaled_workspace_bytes.restype = sz
    lib.goom_count_nonfinite.argtypes = [vp, vp, sz, i32, vp]
    lib.goom_to_goom_backward.argtypes = [vp, vp, vp, vp, sz, i32, C.c_double]
    lib.goom_from_goom_backward.argtypes = [vp, vp, vp, vp, sz, i32, C.c_double]
    lib.goom_affine_scan_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, i64, i32, po, vp, sz]
    lib.goom_affine_scan_backward_workspace_bytes.argtypes = [i64, i32, i64, i32, po]
    lib.goom_affine_scan_backward_workspace_bytes.restype = sz
    lib.goom_lmme_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, u32, vp, sz]
    lib.goom_lmme_backward_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, u32]
    lib.goom_lmme_backward_workspace_bytes.restype = sz
    lib.goom_scaled_exp_backward.argtypes = [vp, vp, vp, vp, sz, i32]
    lib.goom_scan_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i64, i32, po, vp, sz]
    lib.goom_scan_backward_workspace_bytes.argtypes = [i64, i32, i32, i64, i32, po, i32]
    lib.goom_scan_backward_workspace_bytes.restype = sz
    _lib = lib
    return lib


class GoomErrorNoLib(RuntimeError):
    def __init__(self):
        super().__init__(f"{_LIB_PATH} is not built; run __graft_entry__.build() (hipcc, gfx950). "
                         "There is no CPU fallback.")


def status_name(status: int) -> str:
    return load_library().goom_status_name(status).decode()


def _dtype_code(t):
    import torch
    if t.dtype in (torch.complex64, torch.float32):
        return C64
    if t.dtype in (torch.complex128, torch.float64):
        return C128
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libgoom takes contiguous device tensors")
    return C.c_void_p(t.data_ptr())


class Goom:
    """A libgoom context on one device, bound to torch's current stream at creation (or
    to ``stream``).  Methods mirror the C entry points and allocate outputs/workspaces
    with torch."""

    def __init__(self, device: int = 0, stream=None):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.device = torch.device("cuda", device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        self._stream = stream
        self._ctx = C.c_void_p()
        st = self.lib.goom_create(C.byref(self._ctx), device, C.c_void_p(stream.cuda_stream))
        if st != 0:
            raise GoomError(st, self.lib.goom_last_error(None).decode())
        self._ws = None

    def close(self):
        if self._ctx:
            self.lib.goom_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != 0:
            raise GoomError(st, self.lib.goom_last_error(self._ctx).decode())

    def set_stream(self, stream):
        self._stream = stream
        self._check(self.lib.goom_set_stream(self._ctx, C.c_void_p(stream.cuda_stream)))

    def probe_bandwidth(self, a, b, mode: int):
        """One streaming pass (0 read a, 1 fill b, 2 copy a to b) on the context's stream; the caller times it."""
        nbytes = b.numel() * b.element_size()
        self._check(self.lib.goom_probe_bandwidth(self._ctx, _ptr(a), _ptr(b), nbytes, mode))

    PROBE_MATRIX_FLOP_PER_ITER = 134217728

    def probe_matrix_unit(self, sink, iters: int, double: bool = False):
        """A kernel of nothing but matrix instructions (PROBE_MATRIX_FLOP_PER_ITER * iters flop) on the context's
        stream; sink: a device tensor of at least 4 bytes; the caller times it."""
        self._check(self.lib.goom_probe_matrix_unit(self._ctx, _ptr(sink), iters, 1 if double else 0))

    def profile_enable(self, on: bool = True):
        self._check(self.lib.goom_profile_enable(self._ctx, int(on)))

    def profile_records(self):
        """[(label, milliseconds)] for the kernels of the last compute call (waits for them)."""
        out = []
        for i in range(self.lib.goom_profile_count(self._ctx)):
            label, ms = C.c_char_p(), C.c_float()
            self._check(self.lib.goom_profile_get(self._ctx, i, C.byref(label), C.byref(ms)))
            out.append((label.value.decode(), float(ms.value)))
        return out

    def workspace(self, nbytes: int):
        """A cached 256-byte aligned scratch tensor of at least nbytes (None for 0)."""
        if nbytes == 0:
            return None, 0
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = self.torch.empty(nbytes, dtype=self.torch.uint8, device=self.device)
        return self._ws, self._ws.numel()

    # ---- codecs
    def to_goom(self, x, flags: int = ZERO_NEG_INF, out=None):
        torch = self.torch
        code = _dtype_code(x)
        if out is None:
            out = torch.empty(x.shape, dtype=torch.complex64 if code == C64 else torch.complex128, device=x.device)
        self._check(self.lib.goom_to_goom(self._ctx, _ptr(x), _ptr(out), x.numel(), code, flags))
        return out

    def from_goom(self, y, out=None):
        torch = self.torch
        code = _dtype_code(y)
        if out is None:
            out = torch.empty(y.shape, dtype=torch.float32 if code == C64 else torch.float64, device=y.device)
        self._check(self.lib.goom_from_goom(self._ctx, _ptr(y), _ptr(out), y.numel(), code))
        return out

    # ---- LMME
    def lmme(self, a, b, flags: int = LMME_FAST, out=None):
        torch = self.torch
        code = _dtype_code(a)
        n, d = a.shape[-2:]
        d2, m = b.shape[-2:]
        assert d == d2 and a.shape[:-2] == b.shape[:-2] and a.dtype == b.dtype
        batch = 1
        for s in a.shape[:-2]:
            batch *= s
        if out is None:
            out = torch.empty(a.shape[:-2] + (n, m), dtype=a.dtype, device=a.device)
        ws, wsn = self.workspace(self.lib.goom_lmme_workspace_bytes(batch, n, d, m, code, flags))
        self._check(self.lib.goom_lmme(self._ctx, _ptr(a), _ptr(b), _ptr(out), batch, n, d, m, code, flags,
                                       _ptr(ws), wsn))
        return out

    # ---- scans
    def _scan_shapes(self, mats, init):
        T, d, d2 = mats.shape[-3:]
        assert d == d2
        lead = mats.shape[:-3]
        batch = 1
        for s in lead:
            batch *= s
        if init is not None:
            assert init.shape[:-2] == lead and init.shape[-2] == d and init.dtype == mats.dtype
            m = init.shape[-1]
        else:
            m = d
        return lead, batch, T, d, m

    def scan(self, mats, init=None, chunk_len: int = 0, out=None):
        torch = self.torch
        code = _dtype_code(mats)
        lead, batch, T, d, m = self._scan_shapes(mats, init)
        opts = ScanOpts(chunk_len, 0)
        if out is None:
            out = torch.empty(lead + (T, d, m), dtype=mats.dtype, device=mats.device)
        ws, wsn = self.workspace(self.lib.goom_scan_workspace_bytes(T, d, m, batch, code, C.byref(opts)))
        self._check(self.lib.goom_scan(self._ctx, _ptr(mats), _ptr(init), _ptr(out), T, d, m, batch, code,
                                       C.byref(opts), _ptr(ws), wsn))
        return out

    STATIC_SCRATCH_BYTES = 40 << 20

    def scan_static(self, mats, out, init=None, chunk_len: int = 0):
        """goom_scan_static: the scan with the library's static scratch array as its workspace.  `out` is the
        caller's; nothing is allocated here or in the library."""
        code = _dtype_code(mats)
        lead, batch, T, d, m = self._scan_shapes(mats, init)
        assert tuple(out.shape) == tuple(lead + (T, d, m)) and out.dtype == mats.dtype
        opts = ScanOpts(chunk_len, 0)
        self._check(self.lib.goom_scan_static(self._ctx, _ptr(mats), _ptr(init), _ptr(out), T, d, m, batch, code,
                                              C.byref(opts)))
        return out

    def reduce(self, mats, init=None, chunk_len: int = 0, out=None):
        torch = self.torch
        code = _dtype_code(mats)
        lead, batch, T, d, m = self._scan_shapes(mats, init)
        opts = ScanOpts(chunk_len, 0)
        if out is None:
            out = torch.empty(lead + (d, m), dtype=mats.dtype, device=mats.device)
        ws, wsn = self.workspace(self.lib.goom_reduce_workspace_bytes(T, d, m, batch, code, C.byref(opts)))
        self._check(self.lib.goom_reduce(self._ctx, _ptr(mats), _ptr(init), _ptr(out), T, d, m, batch, code,
                                         C.byref(opts), _ptr(ws), wsn))
        return out

    def scan_real(self, x, init=None, chunk_len: int = 0, out=None, final_only: bool = False):
        """Prefix products (or, with final_only, the last one) of real matrices x: [..., T, d, d], as GOOMs."""
        torch = self.torch
        ctype = torch.complex64 if x.dtype == torch.float32 else torch.complex128
        code = C64 if x.dtype == torch.float32 else C128
        T, d = x.shape[-3], x.shape[-1]
        lead = x.shape[:-3]
        m = d if init is None else init.shape[-1]
        batch = 1
        for s in lead:
            batch *= s
        opts = ScanOpts(chunk_len, 0)
        if out is None:
            out = torch.empty(lead + ((d, m) if final_only else (T, d, m)), dtype=ctype, device=x.device)
        if final_only:
            ws, wsn = self.workspace(self.lib.goom_reduce_real_workspace_bytes(T, d, m, batch, code, C.byref(opts)))
            self._check(self.lib.goom_reduce_real(self._ctx, _ptr(x), _ptr(init), _ptr(out), T, d, m, batch, code,
                                                  C.byref(opts), _ptr(ws), wsn))
        else:
            ws, wsn = self.workspace(self.lib.goom_scan_real_workspace_bytes(T, d, m, batch, code, C.byref(opts)))
            self._check(self.lib.goom_scan_real(self._ctx, _ptr(x), _ptr(init), _ptr(out), T, d, m, batch, code,
                                                C.byref(opts), _ptr(ws), wsn))
        return out

    def affine_scan(self, a, bias, h0=None, chunk_len: int = 0, out=None, time_invariant: bool = False):
        """h_t = A_t h_{t-1} + bias_t.  a: [..., T, d, d], or [..., d, d] with time_invariant=True."""
        torch = self.torch
        code = _dtype_code(a)
        T, d = bias.shape[-2:]
        lead = bias.shape[:-2]
        assert a.shape == (lead + (d, d) if time_invariant else lead + (T, d, d)) and a.dtype == bias.dtype
        batch = 1
        for s in lead:
            batch *= s
        opts = ScanOpts(chunk_len, AFFINE_TIME_INVARIANT if time_invariant else 0)
        if out is None:
            out = torch.empty(lead + (T, d), dtype=a.dtype, device=a.device)
        ws, wsn = self.workspace(self.lib.goom_affine_scan_workspace_bytes(T, d, batch, code, C.byref(opts)))
        self._check(self.lib.goom_affine_scan(self._ctx, _ptr(a), _ptr(bias), _ptr(h0), _ptr(out), T, d, batch,
                                              code, C.byref(opts), _ptr(ws), wsn))
        return out

    def affine_scan_scaled(self, a, bias, h0=None, chunk_len: int = 0, time_invariant: bool = False,
                           want_logscale: bool = False):
        """The recurrence's states as exp(h - max Re h + 2), real, and optionally the log scales."""
        torch = self.torch
        code = _dtype_code(a)
        T, d = bias.shape[-2:]
        lead = bias.shape[:-2]
        assert a.shape == (lead + (d, d) if time_invariant else lead + (T, d, d)) and a.dtype == bias.dtype
        batch = 1
        for s in lead:
            batch *= s
        opts = ScanOpts(chunk_len, AFFINE_TIME_INVARIANT if time_invariant else 0)
        comp = torch.float32 if a.dtype == torch.complex64 else torch.float64
        out = torch.empty(lead + (T, d), dtype=comp, device=a.device)
        c = torch.empty(lead + (T,), dtype=comp, device=a.device) if want_logscale else None
        ws, wsn = self.workspace(self.lib.goom_affine_scan_scaled_workspace_bytes(T, d, batch, code, C.byref(opts)))
        self._check(self.lib.goom_affine_scan_scaled(self._ctx, _ptr(a), _ptr(bias), _ptr(h0), _ptr(out), _ptr(c), T, d,
                                                     batch, code, C.byref(opts), _ptr(ws), wsn))
        return (out, c) if want_logscale else out

    def scan_reset(self, jac, s0=None, chunk_len: int = 0, policy: int = RESET_ALWAYS,
                   cos_threshold: float = 0.99, want_states: bool = True):
        torch = self.torch
        code = _dtype_code(jac)
        T, d, _ = jac.shape[-3:]
        lead = jac.shape[:-3]
        batch = 1
        for s in lead:
            batch *= s
        opts = ResetOpts(chunk_len, policy, cos_threshold)
        states = torch.empty(lead + (T, d, d), dtype=jac.dtype, device=jac.device)
        flags = torch.zeros(lead + (T,), dtype=torch.uint8, device=jac.device)
        growth = torch.zeros(lead + (d,), dtype=torch.float64, device=jac.device)
        ws, wsn = self.workspace(self.lib.goom_scan_reset_workspace_bytes(T, d, batch, code, C.byref(opts)))
        self._check(self.lib.goom_scan_reset(self._ctx, _ptr(jac), _ptr(s0), _ptr(states), _ptr(flags), _ptr(growth),
                                             T, d, batch, code, C.byref(opts), _ptr(ws), wsn))
        return states, flags, growth

    def scan_reset_tree(self, jac, s0=None, policy: int = RESET_COLINEAR, cos_threshold: float = 0.99):
        """The selective-resetting scan in the order of the paper's parallel prefix scan; returns (states, flags)."""
        torch = self.torch
        code = _dtype_code(jac)
        T, d, _ = jac.shape[-3:]
        lead = jac.shape[:-3]
        batch = 1
        for s in lead:
            batch *= s
        opts = ResetOpts(0, policy, cos_threshold)
        states = torch.empty(lead + (T, d, d), dtype=jac.dtype, device=jac.device)
        flags = torch.zeros(lead + (T,), dtype=torch.uint8, device=jac.device)
        ws, wsn = self.workspace(self.lib.goom_scan_reset_tree_workspace_bytes(T, d, batch, code))
        self._check(self.lib.goom_scan_reset_tree(self._ctx, _ptr(jac), _ptr(s0), _ptr(states), _ptr(flags), T, d, batch, code,
                                                  C.byref(opts), _ptr(ws), wsn))
        return states, flags

    def lyapunov_spectrum(self, jac, dt: float, s0=None, chunk_len: int = 0, policy: int = RESET_ALWAYS,
                          cos_threshold: float = 0.99):
        torch = self.torch
        code = _dtype_code(jac)
        T, d, _ = jac.shape[-3:]
        lead = jac.shape[:-3]
        batch = 1
        for s in lead:
            batch *= s
        opts = ResetOpts(chunk_len, policy, cos_threshold)
        lam = torch.zeros(lead + (d,), dtype=torch.float64, device=jac.device)
        ws, wsn = self.workspace(self.lib.goom_scan_reset_workspace_bytes(T, d, batch, code, C.byref(opts)))
        self._check(self.lib.goom_lyapunov_spectrum(self._ctx, _ptr(jac), _ptr(s0), None, _ptr(lam), T, d, dt, batch,
                                                    code, C.byref(opts), _ptr(ws), wsn))
        return lam

    def lyapunov_spectrum_per_step(self, jac, dt: float, s0=None, chunk_len: int = 0, policy: int = RESET_ALWAYS,
                                   cos_threshold: float = 0.99, want_step_logs: bool = False):
        """Spectrum by the four groups of parallel computations (two QRs per step)."""
        torch = self.torch
        code = _dtype_code(jac)
        T, d, _ = jac.shape[-3:]
        lead = jac.shape[:-3]
        batch = 1
        for s in lead:
            batch *= s
        opts = ResetOpts(chunk_len, policy, cos_threshold)
        lam = torch.zeros(lead + (d,), dtype=torch.float64, device=jac.device)
        logs = torch.zeros(lead + (T, d), dtype=torch.float64, device=jac.device) if want_step_logs else None
        ws, wsn = self.workspace(self.lib.goom_lyapunov_spectrum_per_step_workspace_bytes(
            T, d, batch, code, C.byref(opts), 0, 1 if want_step_logs else 0))
        self._check(self.lib.goom_lyapunov_spectrum_per_step(self._ctx, _ptr(jac), _ptr(s0), None, _ptr(logs), _ptr(lam),
                                                             T, d, dt, batch, code, C.byref(opts), _ptr(ws), wsn))
        return (lam, logs) if want_step_logs else lam

    def largest_lyapunov(self, jac, dt: float, u0=None, chunk_len: int = 0):
        """Largest exponent as LSE(2 v') / (2 dt T), v' = J_T ... J_1 u_0 over GOOMs."""
        torch = self.torch
        code = _dtype_code(jac)
        T, d, _ = jac.shape[-3:]
        lead = jac.shape[:-3]
        batch = 1
        for s in lead:
            batch *= s
        opts = ScanOpts(chunk_len, 0)
        lle = torch.zeros(lead, dtype=torch.float64, device=jac.device)
        ws, wsn = self.workspace(self.lib.goom_largest_lyapunov_workspace_bytes(T, d, batch, code, C.byref(opts)))
        self._check(self.lib.goom_largest_lyapunov(self._ctx, _ptr(jac), _ptr(u0), _ptr(lle), T, d, dt, batch, code,
                                                   C.byref(opts), _ptr(ws), wsn))
        return lle

    def count_nonfinite(self, z) -> int:
        """Entries of a GOOM tensor whose log-magnitude is +inf or NaN (synchronises to return the number)."""
        cnt = self.torch.zeros(1, dtype=self.torch.int64, device=z.device)
        self._check(self.lib.goom_count_nonfinite(self._ctx, _ptr(z), z.numel(), _dtype_code(z), _ptr(cnt)))
        return int(cnt.item())

    def to_goom_backward(self, x, grad_re, eps: float):
        """grad_re * s(x) / (|x| + eps): backward of to_goom with the paper's redefined derivatives."""
        out = self.torch.empty_like(x)
        self._check(self.lib.goom_to_goom_backward(self._ctx, _ptr(x), _ptr(grad_re), _ptr(out), x.numel(), _dtype_code(x), eps))
        return out

    def from_goom_backward(self, y, grad_x, eps: float):
        """grad_x * (x + s(x) eps): backward of from_goom with the paper's redefined derivative."""
        out = self.torch.empty_like(grad_x)
        self._check(self.lib.goom_from_goom_backward(self._ctx, _ptr(y), _ptr(grad_x), _ptr(out), y.numel(), _dtype_code(y), eps))
        return out

    def affine_scan_backward(self, a, bias, h, grad_h, h0=None, chunk_len: int = 0, time_invariant: bool = False):
        """Gradients of a loss with respect to the log-magnitudes of a, bias (and h0), given grad_h = dL / d Re h.
        time_invariant: a is [..., d, d], one matrix for all steps, and so is its gradient."""
        torch = self.torch
        code = _dtype_code(a)
        T, d = bias.shape[-2:]
        lead = bias.shape[:-2]
        batch = 1
        for s in lead:
            batch *= s
        comp = torch.float32 if a.dtype == torch.complex64 else torch.float64
        ashape = lead + ((d, d) if time_invariant else (T, d, d))
        assert a.shape == ashape and h.shape == bias.shape and grad_h.shape == bias.shape and grad_h.dtype == comp
        opts = ScanOpts(chunk_len, AFFINE_TIME_INVARIANT if time_invariant else 0)
        ga = torch.empty(ashape, dtype=comp, device=a.device)
        gb = torch.empty(lead + (T, d), dtype=comp, device=a.device)
        gh0 = torch.empty(lead + (d,), dtype=comp, device=a.device) if h0 is not None else None
        ws, wsn = self.workspace(self.lib.goom_affine_scan_backward_workspace_bytes(T, d, batch, code, C.byref(opts)))
        self._check(self.lib.goom_affine_scan_backward(self._ctx, _ptr(a), _ptr(bias), _ptr(h0), _ptr(h), _ptr(grad_h), _ptr(ga), _ptr(gb),
                                                       _ptr(gh0), T, d, batch, code, C.byref(opts), _ptr(ws), wsn))
        return ga, gb, gh0

    def lmme_backward(self, a, b, c, grad_c, flags: int = LMME_FAST):
        """Gradients of a loss with respect to the log-magnitudes of a and b, given c = lmme(a, b) and grad_c = dL / d Re c."""
        torch = self.torch
        code = _dtype_code(a)
        n, d = a.shape[-2:]
        m = b.shape[-1]
        lead = a.shape[:-2]
        batch = 1
        for s in lead:
            batch *= s
        comp = torch.float32 if a.dtype == torch.complex64 else torch.float64
        assert b.shape == lead + (d, m) and c.shape == lead + (n, m) and grad_c.shape == c.shape
        assert b.dtype == a.dtype and c.dtype == a.dtype and grad_c.dtype == comp
        ga = torch.empty(lead + (n, d), dtype=comp, device=a.device)
        gb = torch.empty(lead + (d, m), dtype=comp, device=a.device)
        ws, wsn = self.workspace(self.lib.goom_lmme_backward_workspace_bytes(batch, n, d, m, code, flags))
        self._check(self.lib.goom_lmme_backward(self._ctx, _ptr(a), _ptr(b), _ptr(c), _ptr(grad_c), _ptr(ga), _ptr(gb), batch, n, d, m, code,
                                                flags, _ptr(ws), wsn))
        return ga, gb

    def scan_backward(self, mats, p, grad_p, init=None, chunk_len: int = 0):
        """Gradients of a loss with respect to the log-magnitudes of the factors (and of init), given the scan's states p and
        grad_p = dL / d Re p."""
        torch = self.torch
        code = _dtype_code(mats)
        lead, batch, T, d, m = self._scan_shapes(mats, init)
        comp = torch.float32 if mats.dtype == torch.complex64 else torch.float64
        assert p.shape == lead + (T, d, m) and grad_p.shape == p.shape and p.dtype == mats.dtype and grad_p.dtype == comp
        opts = ScanOpts(chunk_len, 0)
        gm = torch.empty(lead + (T, d, d), dtype=comp, device=mats.device)
        gi = torch.empty(lead + (d, m), dtype=comp, device=mats.device) if init is not None else None
        ws, wsn = self.workspace(self.lib.goom_scan_backward_workspace_bytes(T, d, m, batch, code, C.byref(opts), int(init is not None)))
        self._check(self.lib.goom_scan_backward(self._ctx, _ptr(mats), _ptr(init), _ptr(p), _ptr(grad_p), _ptr(gm), _ptr(gi), T, d, m, batch, code,
                                                C.byref(opts), _ptr(ws), wsn))
        return gm, gi

    def scaled_exp(self, z, want_logscale: bool = False):
        """Scaled exponentiation over the last axis: exp(z - max Re z + 2), real."""
        torch = self.torch
        code = _dtype_code(z)
        d = z.shape[-1]
        nvec = z.numel() // d
        comp = torch.float32 if z.dtype == torch.complex64 else torch.float64
        out = torch.empty(z.shape, dtype=comp, device=z.device)
        c = torch.empty(z.shape[:-1], dtype=comp, device=z.device) if want_logscale else None
        self._check(self.lib.goom_scaled_exp(self._ctx, _ptr(z), _ptr(out), _ptr(c), nvec, d, code))
        return (out, c) if want_logscale else out

    def scaled_exp_backward(self, scaled, grad_scaled):
        """Gradient with respect to Re z of scaled = scaled_exp(z), the log-scaling constant detached."""
        assert scaled.shape == grad_scaled.shape and scaled.dtype == grad_scaled.dtype
        out = self.torch.empty_like(scaled)
        self._check(self.lib.goom_scaled_exp_backward(self._ctx, _ptr(scaled), _ptr(grad_scaled), _ptr(out), scaled.numel(), _dtype_code(scaled)))
        return out

    def log_add_exp(self, x, y, out=None):
        """Elementwise GOOM of exp(x) + exp(y)."""
        assert x.shape == y.shape and x.dtype == y.dtype
        if out is None:
            out = self.torch.empty_like(x)
        self._check(self.lib.goom_log_add_exp(self._ctx, _ptr(x), _ptr(y), _ptr(out), x.numel(), _dtype_code(x)))
        return out
