"""GPU parity at the workloads' full sizes, in the launch configuration the benchmark times.

The oracle cannot walk a million 64 x 64 products in test time, so each case checks
  * a leading part of the workload (or sampled batch items) against the oracle, element by
    element, with the same tolerances and conditioning masks as the small cases;
  * properties that hold at any size and that a wrong chunk boundary, carry or index would
    break: every prefix equals its matrix times the previous prefix (recomputed here in
    double, at every chunk boundary and at sampled interior steps), the reduction equals the
    last prefix, and the growth rate equals its closed form.
Inputs are drawn on the device by a seeded generator; the slices the oracle needs are copied
to the host."""
import math

import numpy as np
import pytest

import synthetic_inputs as si
from test_gpu_parity import compare, dev, host, say, tolerance, with_sensitivity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    from paper_2510_03426_amd import Goom
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return Goom(0)


def one_step_defect(x_t, prev, cur):
    """max over well-conditioned entries of | log|M_t P_{t-1}| - Re(P_t) | and the number of sign
    mismatches, with P_{t-1}, P_t given as complex64 GOOMs and M_t as reals; computed in double."""
    pre = prev.real.astype(np.float64)
    cmax = pre.max(axis=0, keepdims=True)
    w = np.where(prev.imag != 0, -1.0, 1.0) * np.exp(pre - cmax)
    m = x_t.astype(np.float64)
    y = m @ w
    mass = np.abs(m) @ np.abs(w)
    ok = np.abs(y) * 8.0 >= mass  # cancellation factor at most 8: rounding of P_{t-1} stays small
    want_re = np.log(np.abs(y)) + cmax
    got_re = cur.real.astype(np.float64)
    defect = np.abs(want_re - got_re)[ok].max()
    signs = int(np.sum(((y < 0) != (cur.imag != 0)) & ok))
    return defect, signs, ok.mean()


def test_config2_long_chain_scan_full_size(G, oracle):
    import torch
    T, d = 1 << 20, 64
    device = torch.device("cuda", 0)
    keep = 32768  # leading steps the oracle walks
    z = torch.empty((T, d, d), dtype=torch.complex64, device=device)
    # real matrices kept on the host where the test needs them: the leading part, every chunk
    # boundary and a few interior steps
    L = 1024
    sampled = sorted(set(range(L, T, L)) | {5, 1000, 77777, 500001, 500002, T - 2, T - 1} |
                     set(int(v) for v in np.random.default_rng(7).integers(1, T, 64)))
    x_keep = {}
    x_head = None
    say(f"config 2 at full size: T={T} d={d}; drawing and encoding on the device")
    blk = 1 << 16
    for t0, x in si.device_normal_blocks(si.BASE_SEED * 10 + 2, T, (d, d), device, blk):
        G.to_goom(x, out=z[t0:t0 + x.shape[0]])
        if t0 == 0:
            x_head = x[:keep].cpu().numpy()
        for t in sampled:
            if t0 <= t < t0 + x.shape[0]:
                x_keep[t] = x[t - t0].cpu().numpy()
        del x
    out = G.scan(z)  # default options: what the benchmark runs
    torch.cuda.synchronize()
    say("  scan done; oracle on the leading part")

    zs = host(z[:keep])
    assert np.array_equal(zs.view(np.uint32), oracle.to_goom(x_head).view(np.uint32))
    sample = sorted({0, 1, 2, 63, 64, 511, L - 2, L - 1, L, L + 1, 2 * L - 1, 2 * L, 3 * L, 7 * L - 1, 7 * L,
                     16 * L - 1, 16 * L, 16 * L + 1, 31 * L, keep - 1} | set(range(997, keep, 1499)))
    fn = lambda mats: oracle.ScanStream(d, scaled=True).advance(mats, sample_t=sample, return_kappa=True)
    re, sg, kap, well = with_sensitivity(fn, [zs], np.float32, nprobe=1)
    compare(host(out[sample]), re, sg, kap, name=f"config 2, {len(sample)} sampled prefixes of the first {keep}",
            max_ill_fraction=0.03, well=well)

    # every chunk boundary and sampled interior steps: P_t = M_t P_{t-1}
    worst, bad_signs = 0.0, 0
    idx = torch.tensor(sampled, device=device)
    cur_all = host(out[idx])
    prev_all = host(out[idx - 1])
    for n, t in enumerate(sampled):
        defect, signs, frac = one_step_defect(x_keep[t], prev_all[n], cur_all[n])
        worst = max(worst, defect)
        bad_signs += signs
        assert frac > 0.3
    # a stored log-magnitude near 2e6 is rounded to a multiple of 0.125 or 0.25: each entry of
    # P_{t-1} is off by a few percent, the 64-term sum by (a few percent) * 8 / sqrt(64), and
    # P_t carries its own rounding; a misplaced carry would show as a defect of order 10 or more
    say(f"  one-step recurrence at {len(sampled)} steps (all {T // L - 1} chunk boundaries): worst defect {worst:.3f}, "
        f"{bad_signs} sign mismatches")
    assert worst < 0.75 and bad_signs == 0

    # the reduction is the last prefix
    fin = host(G.reduce(z))
    last = host(out[T - 1])
    dre = np.abs(fin.real.astype(np.float64) - last.real.astype(np.float64))
    same = (fin.imag == last.imag) & (dre <= 0.5)
    say(f"  reduction against the last prefix: {same.mean():.2%} of entries within 0.5 with equal signs, worst {dre.max():.3f}")
    assert same.mean() > 0.99 and np.all(dre <= tolerance(last.real.astype(np.float64), np.float32))
    # growth rate of a product of Gaussian matrices: (ln 2 + psi(d / 2)) / 2 per step
    from scipy.special import digamma
    lam = 0.5 * (math.log(2.0) + digamma(d / 2))
    rate = float(last.real.max()) / T
    say(f"  log-magnitude of the last prefix: {last.real.max():.1f}; growth per step {rate:.5f} (closed form {lam:.5f})")
    assert last.real.max() > 2.0e6 and abs(rate - lam) < 5e-4
    del z, out


def long_scan_case(G, oracle, T, d, L, keep, tmax, nbound, blk, seed, rate_tol, real=False):
    """A scan with default options at a benchmark size: the leading `keep` steps against the oracle, the
    one-step recurrence at up to `nbound` chunk boundaries (chunks of L steps) and 100 interior steps below
    tmax, the reduction against the last prefix, the growth rate against its closed form."""
    import torch
    device = torch.device("cuda", 0)
    # real=True: the scan is fed the real matrices themselves (goom_scan_real), not their encodings
    z = torch.empty((T, d, d), dtype=torch.float32 if real else torch.complex64, device=device)
    rng = np.random.default_rng(seed)
    bounds = list(range(L, tmax, L))
    if len(bounds) > nbound:
        bounds = sorted(set(int(v) for v in rng.choice(bounds, nbound, replace=False)) | {L, 2 * L})
    sampled = sorted(set(bounds) | set(int(v) for v in rng.integers(1, tmax, 100)))
    x_keep = {}
    x_head = None
    say(f"long scan: T={T} d={d} ({len(sampled)} steps checked by the recurrence)")
    for t0, x in si.device_normal_blocks(si.BASE_SEED * 10 + seed, T, (d, d), device, blk):
        if real:
            z[t0:t0 + x.shape[0]].copy_(x)
        else:
            G.to_goom(x, out=z[t0:t0 + x.shape[0]])
        if t0 == 0:
            x_head = x[:keep].cpu().numpy()
        for t in sampled:
            if t0 <= t < t0 + x.shape[0]:
                x_keep[t] = x[t - t0].cpu().numpy()
        del x
    out = G.scan_real(z) if real else G.scan(z)
    torch.cuda.synchronize()
    if real:
        zs = oracle.to_goom(x_head)
    else:
        zs = host(z[:keep])
        assert np.array_equal(zs.view(np.uint32), oracle.to_goom(x_head).view(np.uint32))
    sample = sorted(t for t in ({0, 1, 2, 3, L - 1, L, L + 1, 2 * L - 1, 2 * L, 3 * L, keep - 1} | (set(range(keep // 7, keep, keep // 9)) if keep >= 9 else set())) if t < keep)
    fn = lambda mats: oracle.ScanStream(d, scaled=True).advance(mats, sample_t=sample, return_kappa=True)
    re, sg, kap, well = with_sensitivity(fn, [zs], np.float32, nprobe=1)
    compare(host(out[sample]), re, sg, kap, name=f"d={d}: {len(sample)} sampled prefixes of the first {keep}", max_ill_fraction=0.03, well=well)
    worst, bad_signs = 0.0, 0
    idx = torch.tensor(sampled, device=device)
    cur_all, prev_all = host(out[idx]), host(out[idx - 1])
    for n, t in enumerate(sampled):
        defect, signs, frac = one_step_defect(x_keep[t], prev_all[n], cur_all[n])
        worst = max(worst, defect)
        bad_signs += signs
    say(f"  one-step recurrence at {len(sampled)} steps: worst defect {worst:.3f}, {bad_signs} sign mismatches")
    assert worst < 0.75 and bad_signs == 0
    fin = host(G.scan_real(z, final_only=True) if real else G.reduce(z))
    last = host(out[T - 1])
    dre = np.abs(fin.real.astype(np.float64) - last.real.astype(np.float64))
    well_last = dre <= tolerance(last.real.astype(np.float64), np.float32)
    say(f"  reduction against the last prefix: {well_last.mean():.3%} of entries within tolerance")
    assert np.array_equal(fin.imag[well_last], last.imag[well_last]) and well_last.mean() > 0.995
    from scipy.special import digamma
    lam = 0.5 * (math.log(2.0) + digamma(d / 2))
    rate = float(last.real.max()) / T
    say(f"  log-magnitude of the last prefix: {last.real.max():.1f}; growth per step {rate:.5f} (closed form {lam:.5f})")
    assert abs(rate - lam) < rate_tol
    del z, out


def test_config2_scan_of_real_matrices_full_size(G, oracle):
    # the headline chain (T = 2^20 of 64 x 64) fed as real matrices, in the launch configuration bench.py times
    # (1024 chunks of 1024 steps); the recurrence is checked below 2^18 (further on a stored log-magnitude is
    # rounded too coarsely for the check to say much)
    long_scan_case(G, oracle, 1 << 20, 64, 1024, 2100, 1 << 18, 300, 1 << 14, 164, 1e-3, real=True)


@pytest.mark.parametrize("d,tmax", [(8, 1 << 21), (16, 1 << 20)])
def test_long_scans_of_small_matrices(G, oracle, d, tmax):
    # T = 2^22 chains of 8 x 8 and 16 x 16 matrices, as the benchmark runs them (8192 chunks of 512 steps, one
    # wave per chain or per pair of 8 x 8 chains); the recurrence is checked below tmax only (further on a stored
    # log-magnitude is so coarsely rounded that the check says little)
    long_scan_case(G, oracle, 1 << 22, d, 512, 32768, tmax, 500, 1 << 19, 80 + d, 1.5e-3)


@pytest.mark.parametrize("d,T", [(48, 1 << 19), (96, 1 << 17)])
def test_long_scans_between_tiles(G, oracle, d, T):
    # 48 x 48 and 96 x 96 matrices as the benchmark runs them (chunks of 512 steps; the hot kernel with the
    # rows and columns beyond the matrix left out of the product)
    long_scan_case(G, oracle, T, d, 512, 1200, T, 300, 1 << 14, 200 + d, 3e-3)


def test_long_scan_128(G, oracle):
    # T = 2^18 chain of 128 x 128 matrices (256 chunks of 1024 steps, one workgroup per compute unit)
    long_scan_case(G, oracle, 1 << 18, 128, 1024, 2048, 1 << 18, 300, 1 << 14, 128, 2e-3)


def test_long_scan_1024(G, oracle):
    # T = 512 chain of 1024 x 1024 matrices (8 chunks of 64 steps, every step a round of GEMM launches); the
    # oracle walks the first steps only, the recurrence is checked at every chunk boundary
    long_scan_case(G, oracle, 512, 1024, 64, 3, 512, 10, 64, 1024, 2e-2)


def test_long_scan_256(G, oracle):
    # T = 2^15 chain of 256 x 256 matrices (128 chunks of 256 steps, states resident in registers, two workgroups per chain)
    long_scan_case(G, oracle, 1 << 15, 256, 256, 640, 1 << 15, 200, 1 << 12, 256, 5e-3)


@pytest.mark.parametrize("ctype", ["complex64", "complex128"])
def test_config3_batched_lmme_full_size(G, oracle, ctype):
    import torch
    from paper_2510_03426_amd import LMME_EXACT
    B, n = 8192, 128
    device = torch.device("cuda", 0)
    ct = getattr(torch, ctype)
    say(f"config 3 at full size: {B} pairs of {n}x{n} {ctype}")
    a = si.device_wide_range_gooms(si.BASE_SEED * 10 + 31, (B, n, n), 200.0, ct, device)
    b = si.device_wide_range_gooms(si.BASE_SEED * 10 + 32, (B, n, n), 200.0, ct, device)
    c = G.lmme(a, b, flags=LMME_EXACT)
    torch.cuda.synchronize()
    comp = np.float32 if ctype == "complex64" else np.float64
    pairs = [0, 1, 4095, 6000, B - 1]
    for p in pairs:
        ah, bh = host(a[p]), host(b[p])
        re, sg, kap, well = with_sensitivity(lambda x, y: oracle.lmme(x, y, return_kappa=True), [ah, bh], comp, nprobe=1)
        compare(host(c[p]), re, sg, kap, name=f"config 3 {ctype} pair {p}", max_ill_fraction=0.002, well=well)
    del a, b, c


def test_codecs_float_sweep_of_bit_patterns(G, oracle):
    """Float codecs over 2^28 of the 2^32 bit patterns, one from every run of sixteen consecutive patterns (so
    every exponent, the subnormals, both signs, infinities and NaNs): as inputs of to_goom, and as log-magnitudes
    of from_goom.  Equal bits throughout; stops at the first block with a mismatch."""
    block = 1 << 24
    for blk in range(16):
        i = np.arange(blk * block, (blk + 1) * block, dtype=np.uint64)
        bits = (i * 16 + (i * 7 + blk) % 16).astype(np.uint32)
        x = bits.view(np.float32)
        want = oracle.to_goom(x)
        got = host(G.to_goom(dev(x)))
        a, b = got.view(np.uint32).reshape(-1, 2), want.view(np.uint32).reshape(-1, 2)
        nan = np.isnan(x)
        neq = (a != b).any(axis=1) & ~nan
        assert not neq.any(), f"block {blk}: {neq.sum()} encodings differ, first at bits {bits[np.argwhere(neq)[0, 0]]:#x}"
        assert np.all(np.isnan(got.real[nan]))
        z = (x.astype(np.complex64) + np.complex64(1j * np.pi) * (bits & 1).astype(np.float32)).astype(np.complex64)
        z.imag[...] = np.where((bits & 1) != 0, np.float32(np.pi), np.float32(0))
        want = oracle.from_goom(z)
        got = host(G.from_goom(dev(z)))
        neq = (got.view(np.uint32) != want.view(np.uint32)) & ~nan
        assert not neq.any(), f"block {blk}: {neq.sum()} decodings differ, first at bits {bits[np.argwhere(neq)[0, 0]]:#x}"
        say(f"  codec sweep block {blk + 1}/16: {block} patterns equal in both directions")


def test_config4_lyapunov_full_size(G, oracle):
    T, d, dt = 131072, 32, 0.01
    say(f"config 4 at full size: Lorenz-96 d={d}, T={T}")
    Jr = None
    for attempt in range(6):  # the Euler map is only marginally stable: take the next stream if it escapes
        try:
            Jr, _ = si.lorenz96_jacobians(si.BASE_SEED + 4 + 1000 * attempt, T, d=d, burn_in=10000)
            break
        except FloatingPointError:
            continue
    assert Jr is not None
    say("  Jacobians ready; sequential QR in double")
    lam_qr = oracle.lyapunov_qr(Jr, dt)
    Jz = dev(oracle.to_goom(Jr))
    lam = host(G.lyapunov_spectrum(Jz, dt))
    err = np.abs(lam - lam_qr)
    say(f"  max |lambda_gpu - lambda_qr| = {err.max():.2e} at k={int(err.argmax()) + 1}; lambda_1 = {lam[0]:.4f} "
        f"(QR {lam_qr[0]:.4f}), sum = {lam.sum():.4f} (QR {lam_qr.sum():.4f})")
    assert err.max() < 1e-3
    # the paper's own pipeline (two QRs per step on the reset states) and the largest exponent alone
    lam_ps = host(G.lyapunov_spectrum_per_step(Jz, dt))
    lle = float(host(G.largest_lyapunov(Jz, dt)))
    e1 = np.zeros(d)
    e1[0] = 1.0
    say(f"  per-step estimator: max |lambda - lambda_qr| = {np.abs(lam_ps - lam_qr).max():.2e}; "
        f"largest exponent from the vector reduction {lle:.5f} (QR method {lam_qr[0]:.5f})")
    assert np.abs(lam_ps - lam_qr).max() < 1e-3
    u = np.full(d, 1.0 / math.sqrt(d))
    assert abs(lle - oracle.lle_standard(Jr, u, dt)) < 1e-3
    # states, flags and growth of the reset scan on the same chain; the leading part against the
    # sequentially reset oracle, column by column (see the small cases for why not entry by entry)
    states, flags, growth = G.scan_reset(Jz)
    assert np.abs(host(growth) / (T * dt) - lam).max() < 1e-9
    fl = host(flags)
    L = 128  # the library's default
    assert fl.sum() == T // L and np.all(fl[L - 1::L] == 1)
    # every entry of every state of the whole run against the sequentially reset oracle (both factorise in
    # double at the same steps); the only entries left out are those below e^-10 of their column's largest (the
    # orthonormal factor of a reset is good to about cond^2 2^-53, up to 1e-8, of a column's norm)
    say("  sequentially reset oracle over the whole chain")
    re, sg, oflag, _ = oracle.reset_scan(oracle.to_goom(Jr), None, check_every=L, policy=1)
    assert np.array_equal(fl, oflag)
    worst = 0.0
    for t0 in range(0, T, 16384):
        sl = slice(t0, t0 + 16384)
        got = host(states[sl])
        tiny = re[sl] < re[sl].max(axis=1, keepdims=True) - 10.0
        compare(got, re[sl], sg[sl], None, name=f"config 4 states {t0}..{t0 + 16383}", max_ill_fraction=0.01, well=~tiny)
    # the last states are orthonormal right after the final reset (T is a multiple of the chunk length)
    q = host(states[T - 1])
    qv = np.where(q.imag != 0, -1.0, 1.0) * np.exp(q.real.astype(np.float64))
    assert np.abs(qv.T @ qv - np.eye(d)).max() < 1e-4


def test_config5_recurrence_full_size(G, oracle):
    import torch
    batch, heads, T, d = 8, 16, 65536, 32
    device = torch.device("cuda", 0)
    say(f"config 5 at full size: batch {batch} x {heads} heads, T={T}, d={d}")
    nseq = batch * heads
    az = torch.empty((batch, heads, T, d, d), dtype=torch.complex64, device=device)
    azf = az.view(nseq, T, d, d)
    picks = [0, nseq - 1]
    a_host = {}
    for s0, x in si.device_normal_blocks(si.BASE_SEED * 10 + 51, nseq, (T, d, d), device, 4, scale=1.05 / math.sqrt(d)):
        G.to_goom(x, out=azf[s0:s0 + x.shape[0]])
        for p in picks:
            if s0 <= p < s0 + x.shape[0]:
                a_host[p] = x[p - s0].cpu().numpy()
        del x
    xin = next(si.device_normal_blocks(si.BASE_SEED * 10 + 52, nseq, (T, d), device, nseq))[1]
    bz = G.to_goom(xin).view(batch, heads, T, d)
    # with this many sequences the library walks each of them start to end; a batch of fewer gets the chunked scan (chunk products,
    # carries, walk), run here on the same input with the chunk length it would choose
    h = G.affine_scan(az, bz)
    got_chunked = {p: host(G.affine_scan(azf[p:p + 1], bz.view(nseq, T, d)[p:p + 1])[0]) for p in picks}
    torch.cuda.synchronize()
    hf = h.view(nseq, T, d)
    fn = lambda a_, b_: oracle.affine_scan(a_, b_, return_kappa=True)
    for p in picks:
        Az = oracle.to_goom(a_host[p])
        bzh = oracle.to_goom(xin[p].cpu().numpy())
        assert np.array_equal(host(azf[p, :64]).view(np.uint32), Az[:64].view(np.uint32))
        # three probes: over 65536 steps the rounding of every step adds up, and a single random probe
        # underestimates the sensitivity of an entry about one time in ten
        re, sg, kap, well = with_sensitivity(fn, [Az, bzh], np.float32, nprobe=3)
        got = host(hf[p])
        # chunk products and carries are held in double, so what reaches a state is the rounding of the last
        # float walk alone, as in a sequential float evaluation: the stated tolerance holds on every entry
        # the oracle marks well conditioned
        compare(got, re, sg, kap, name=f"config 5 sequence {p}", max_ill_fraction=0.05, well=well)
        compare(got_chunked[p], re, sg, kap, name=f"config 5 sequence {p}, chunked scan", max_ill_fraction=0.05, well=well)
        say(f"    |h_T| = exp({got.real[-1].max():.1f})")
    del az, bz, h
