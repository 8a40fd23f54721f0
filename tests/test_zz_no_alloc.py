"""The allocation-free scan entry point (mamba_scan_fwd_static) against mamba_scan_fwd: same kernels, chunk states in
the library's own device buffer instead of a caller's workspace.  Two calls in a row, the second on a smaller input
(the buffer keeps the first call's contents), each compared bit for bit with the existing entry point and, through
it, within tolerance with the oracle."""
import sys

import numpy as np
import pytest
import torch

from paper_2506_01206_amd import synth
from gpu_util import DEV, TOL, assert_close, dev_case, oracle_scan, to_host, values

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def m():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2506_01206_amd import binding
    return binding


def both(m, c, h0=None, chunk_len=0):
    d = dev_case(c)
    args = (d["x"], d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"])
    ref_out, ref_h = m.mamba_scan_fwd(*args, h0=h0, chunk_len=chunk_len)
    out = torch.full_like(ref_out, float("nan"))
    hf = torch.full_like(ref_h, float("nan"))
    m.mamba_scan_fwd_static(*args, h0, out, hf, chunk_len=chunk_len)
    torch.cuda.synchronize()
    return (out, hf), (ref_out, ref_h)


@pytest.mark.parametrize("io", [synth.BF16, synth.F32])
def test_static_scratch_scan_matches_the_workspace_scan(m, io):
    print("\n[gpu-case] static-scratch scan, io=%s" % io, flush=True)
    sys.stdout.flush()
    tol = TOL[io]
    # first call: 3 rows x 5000 tokens x 192 channels, cut into many chunks; second: smaller and shorter chunks
    for (B, L, D, N, cl, seed) in ((3, 5000, 192, 16, 0, 901), (1, 700, 66, 8, 48, 902)):
        c = synth.prefill_case(B, L, D, N, 4, io, seed=seed, random_A=True)
        need = m.mamba_scan_workspace_bytes(B, L, D, N, cl)
        assert 0 < need <= m.MAMBA_SCAN_STATIC_BYTES, need                    # the scratch buffer is in use
        h0 = torch.from_numpy(np.random.default_rng(seed).standard_normal((B, D, N)).astype(np.float32)).to(DEV)
        (out, hf), (ref_out, ref_h) = both(m, c, h0=h0, chunk_len=cl)
        assert torch.equal(out, ref_out) and torch.equal(hf, ref_h)           # same kernels, same order: same bits
        ro, rh = oracle_scan(c, h0=h0.double().cpu().numpy())
        assert_close(values(to_host(out)), ro, tol, "static scan out")
        assert_close(to_host(hf), rh, tol, "static scan state")
    # one chunk: no scratch needed, still served
    c = synth.prefill_case(2, 40, 64, 16, 4, io, seed=903)
    (out, hf), (ref_out, ref_h) = both(m, c, chunk_len=40)
    assert torch.equal(out, ref_out) and torch.equal(hf, ref_h)


def test_static_scratch_scan_refuses_what_does_not_fit(m):
    print("\n[gpu-case] static-scratch scan, oversize", flush=True)
    B, L, D, N = 4, 8192, 4096, 16
    assert m.mamba_scan_workspace_bytes(B, L, D, N, 64) > m.MAMBA_SCAN_STATIC_BYTES
    x = torch.zeros((B, L, D), dtype=torch.bfloat16, device=DEV)
    bc = torch.zeros((B, L, N), dtype=torch.bfloat16, device=DEV)
    A = -torch.ones((D, N), dtype=torch.float32, device=DEV)
    out = torch.full_like(x, 7.0)
    with pytest.raises(m.MambaError) as e:
        m.mamba_scan_fwd_static(x, x, A, bc, bc, None, None, None, None, out, None, chunk_len=64)
    assert e.value.status == m.STATUS["WORKSPACE"]
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                                            # nothing was launched
