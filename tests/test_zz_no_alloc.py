"""goom_scan_static, the scan for callers that cannot allocate device memory: through the C ABI, its
outputs against goom_scan's (same kernels, same plan: equal bits), on two calls in a row, the second
with a smaller input, then an input whose workspace does not fit the static array."""
import ctypes as C

import numpy as np
import pytest

import synthetic_inputs as si

pytestmark = pytest.mark.gpu


def test_scan_static_matches_scan_on_two_calls_in_a_row():
    import torch
    from paper_2510_03426_amd import Goom
    from paper_2510_03426_amd.binding import GoomError, ScanOpts
    assert torch.cuda.is_available(), "this test needs the MI355X"
    g = Goom(0)
    # (T, d, batch, chunk_len): several chunks with a grouped carry phase, then a smaller, ragged case
    for (T, d, batch, chunk) in ((6000, 64, 2, 24), (777, 32, 1, 16)):
        x = si.normal_chain(si.BASE_SEED + 40 + d, T * batch, d).reshape(batch, T, d, d)
        z = g.to_goom(torch.from_numpy(x).cuda())
        opts = ScanOpts(chunk, 0)
        need = g.lib.goom_scan_workspace_bytes(T, d, d, batch, 0, C.byref(opts))
        assert 0 < need <= g.STATIC_SCRATCH_BYTES
        print(f"goom_scan_static: T={T} d={d} batch={batch} chunk_len={chunk} workspace {need} bytes", flush=True)
        ref = g.scan(z, chunk_len=chunk)
        out = torch.empty_like(ref)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        g.scan_static(z, out, chunk_len=chunk)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        a, b = out.cpu().numpy(), ref.cpu().numpy()
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), \
            f"{np.sum(a.view(np.uint32) != b.view(np.uint32))} words differ from goom_scan"
        assert np.isfinite(a.real).all() and a.real.max() > 100.0  # the outputs are real results, past float range soon
    # a default plan that does not fit the array: the call takes the shortest longer chunks that do
    T, d = 4096, 128
    x = si.normal_chain(si.BASE_SEED + 47, T, d).astype(np.float64)
    z = g.to_goom(torch.from_numpy(x).cuda())
    assert z.dtype == torch.complex128
    assert g.lib.goom_scan_workspace_bytes(T, d, d, 1, 1, C.byref(ScanOpts(0, 0))) > g.STATIC_SCRATCH_BYTES
    L = 8
    while g.lib.goom_scan_workspace_bytes(T, d, d, 1, 1, C.byref(ScanOpts(L, 0))) > g.STATIC_SCRATCH_BYTES:
        L *= 2
    print(f"goom_scan_static: T={T} d={d} complex128, default plan too large, chunk_len {L} fits", flush=True)
    ref = g.scan(z, chunk_len=L)
    out = torch.empty_like(ref)
    g.scan_static(z, out)
    torch.cuda.synchronize()
    a, b = out.cpu().numpy(), ref.cpu().numpy()
    assert np.array_equal(a.view(np.uint64), b.view(np.uint64))
    # a scan whose workspace exceeds the array is refused, with nothing enqueued
    T, d = 1 << 16, 128
    big = torch.empty(1, dtype=torch.complex64, device="cuda")  # never dereferenced: the call fails on the host
    opts = ScanOpts(16, 0)
    assert g.lib.goom_scan_workspace_bytes(T, d, d, 1, 0, C.byref(opts)) > g.STATIC_SCRATCH_BYTES
    st = g.lib.goom_scan_static(g._ctx, C.c_void_p(big.data_ptr()), None, C.c_void_p(big.data_ptr()), T, d, d, 1, 0, C.byref(opts))
    assert st == -3 and "goom_scan_static holds" in g.lib.goom_last_error(g._ctx).decode()
    g.close()
