"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds no GOOM arithmetic: it only draws random numbers and integrates the
Lorenz-96 toy system that supplies Jacobians.  Both the CPU oracle and the GPU library
are fed from here so that they see the same bits.  Every array is a pure function of
its arguments; long arrays are produced in fixed-size blocks, each from its own
counter-based (Philox) stream, so any block can be regenerated on its own.

Workloads (shapes and distributions follow the paper's experiments, Section 4):
  * chains of d x d matrices with i.i.d. N(0, 1) entries (Section 4.1);
  * pairs of GOOM matrices with log-magnitudes N(0, sigma^2) and random signs, a
    stress input for LMME far outside float range (Section 3.2);
  * Jacobians of a forward-Euler Lorenz-96 map along a trajectory (stand-in for the
    dynamical-systems dataset of Section 4.2, which is not available offline);
  * per-token transition matrices and inputs of a non-diagonal linear recurrence
    (Section 4.3).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 251003426
_BLOCK_ELEMS = 1 << 22  # elements drawn per Philox stream


def _stream(seed: int, tag: int, block: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) ^ tag, block]))


def normal_f32(seed: int, tag: int, n: int, start: int = 0, threads: int = 8) -> np.ndarray:
    """n standard normals (float32), elements [start, start + n) of an endless stream
    identified by (seed, tag).  start must be a multiple of the block size (2^22)."""
    assert start % _BLOCK_ELEMS == 0
    out = np.empty((n,), dtype=np.float32)
    nblocks = (n + _BLOCK_ELEMS - 1) // _BLOCK_ELEMS
    b0 = start // _BLOCK_ELEMS

    def fill(i):
        lo = i * _BLOCK_ELEMS
        hi = min(n, lo + _BLOCK_ELEMS)
        _stream(seed, tag, b0 + i).standard_normal(hi - lo, dtype=np.float32, out=out[lo:hi])

    if nblocks <= 1 or threads <= 1:
        for i in range(nblocks):
            fill(i)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nblocks)))
    return out


def normal_chain(seed: int, T: int, d: int, t0: int = 0, threads: int = 8) -> np.ndarray:
    """Matrices M_{t0+1} .. M_{t0+T} of a chain with i.i.d. N(0, 1) float32 entries,
    shape [T, d, d] (Section 4.1).  t0 * d * d must be a multiple of 2^22 (or 0)."""
    return normal_f32(seed, 1, T * d * d, start=t0 * d * d, threads=threads).reshape(T, d, d)


def normal_init(seed: int, d: int, m: int) -> np.ndarray:
    """Initial state S_0 with i.i.d. N(0, 1) float32 entries, shape [d, m]."""
    return normal_f32(seed, 2, d * m).reshape(d, m)


def wide_range_goom_pairs(seed: int, batch: int, n: int, d: int, m: int, sigma: float = 200.0,
                          dtype=np.complex64):
    """Pairs (A', B') of GOOM matrices given directly in log form: real parts N(0, sigma^2),
    imaginary parts 0 or pi with probability 1/2 each.  Shapes [batch, n, d], [batch, d, m]."""
    comp = np.float32 if np.dtype(dtype) == np.complex64 else np.float64
    pi = comp(np.pi)
    outs = []
    for tag, shape in ((3, (batch, n, d)), (4, (batch, d, m))):
        cnt = int(np.prod(shape))
        re = (normal_f32(seed, tag, cnt).astype(np.float64) * sigma).astype(comp)
        bits = np.random.Generator(np.random.Philox(key=[(seed << 8) ^ tag, 1 << 40])).integers(
            0, 2, size=cnt, dtype=np.uint8)
        z = np.empty(shape, dtype=dtype)
        z.real = re.reshape(shape)
        z.imag = (bits.astype(comp) * pi).reshape(shape)
        outs.append(z)
    return outs[0], outs[1]


def lorenz96_jacobians(seed: int, T: int, d: int = 32, forcing: float = 8.0, dt: float = 0.01,
                       burn_in: int = 10000):
    """Forward-Euler Lorenz-96: x <- x + dt f(x), f_i = (x_{i+1} - x_{i-2}) x_{i-1} - x_i + F,
    indices cyclic, x_0 = F + N(0, 0.01^2).  After burn_in steps, returns the float32
    Jacobians of the Euler map, J_t = I + dt Df(x_{t-1}), t = 1..T, shape [T, d, d], and
    the float64 trajectory [T + 1, d] they were taken along (x_{t-1} is row t - 1)."""
    rng = _stream(seed, 5, 0)
    x = forcing + 0.01 * rng.standard_normal(d)

    def f(v):
        return (np.roll(v, -1) - np.roll(v, 2)) * np.roll(v, 1) - v + forcing

    traj = np.empty((T + 1, d), dtype=np.float64)
    with np.errstate(over="ignore", invalid="ignore"):  # an escaping trajectory is reported below
        for _ in range(burn_in):
            x = x + dt * f(x)
        traj[0] = x
        for t in range(T):
            x = x + dt * f(x)
            traj[t + 1] = x
    if not np.all(np.isfinite(traj)) or np.abs(traj).max() > 1e3:
        raise FloatingPointError("Lorenz-96 trajectory left the attractor (Euler step too large)")
    xs = traj[:-1]
    J = np.zeros((T, d, d), dtype=np.float64)
    idx = np.arange(d)
    # d f_i / d x_{i+1} = x_{i-1};  d f_i / d x_{i-2} = -x_{i-1};
    # d f_i / d x_{i-1} = x_{i+1} - x_{i-2};  d f_i / d x_i = -1
    J[:, idx, (idx + 1) % d] += xs[:, (idx - 1) % d]
    J[:, idx, (idx - 2) % d] += -xs[:, (idx - 1) % d]
    J[:, idx, (idx - 1) % d] += xs[:, (idx + 1) % d] - xs[:, (idx - 2) % d]
    J[:, idx, idx] += -1.0
    J *= dt
    J[:, idx, idx] += 1.0
    return J.astype(np.float32), traj


def recurrence_inputs(seed: int, batch: int, T: int, d: int, gain: float = 1.05, seq0: int = 0,
                      threads: int = 8):
    """Transition matrices A_t with entries gain * N(0, 1/d) and inputs b_t ~ N(0, 1)^d for
    sequences seq0 .. seq0 + batch - 1 (Section 4.3 shapes).  Returns float32 arrays
    A [batch, T, d, d] and b [batch, T, d].  Each sequence has its own stream."""
    A = np.empty((batch, T, d, d), dtype=np.float32)
    b = np.empty((batch, T, d), dtype=np.float32)
    scale = np.float32(gain / np.sqrt(d))

    def fill(q):
        s = seq0 + q
        A[q] = normal_f32(seed, 1000 + 2 * s, T * d * d, threads=1).reshape(T, d, d) * scale
        b[q] = normal_f32(seed, 1001 + 2 * s, T * d, threads=1).reshape(T, d)

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, range(batch)))
    return A, b


# ------------------------------------------------------------------ device-side draws
# The full-size workloads (tens of GB) are drawn on the GPU by torch's seeded generator; the
# slices the CPU oracle needs are copied to the host, so both sides still see the same bits.

def device_generator(seed: int, device):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    return gen


def device_normal_blocks(seed: int, n_items: int, item_shape, device, block_items: int, scale: float = 1.0):
    """Yield (first_item, float32 tensor [k, *item_shape]) blocks of i.i.d. N(0, scale^2) draws
    covering items [0, n_items); the sequence is a pure function of (seed, block_items)."""
    import torch
    gen = device_generator(seed, device)
    for i0 in range(0, n_items, block_items):
        k = min(block_items, n_items - i0)
        x = torch.randn((k,) + tuple(item_shape), dtype=torch.float32, device=device, generator=gen)
        if scale != 1.0:
            x.mul_(scale)
        yield i0, x


def device_wide_range_gooms(seed: int, shape, sigma: float, ctype, device):
    """GOOM tensor with log-magnitudes N(0, sigma^2) and phases 0 or pi with probability 1/2."""
    import math
    import torch
    gen = device_generator(seed, device)
    comp = torch.float32 if ctype == torch.complex64 else torch.float64
    z = torch.empty(tuple(shape), dtype=ctype, device=device)
    zr = torch.view_as_real(z)
    zr[..., 0] = torch.randn(tuple(shape), dtype=comp, device=device, generator=gen) * sigma
    zr[..., 1] = (torch.rand(tuple(shape), dtype=torch.float32, device=device, generator=gen) < 0.5).to(comp) * \
        torch.tensor(math.pi, dtype=comp).item()
    return z
