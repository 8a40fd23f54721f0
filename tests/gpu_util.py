"""Helpers for the GPU parity tests: moving seeded numpy inputs to the device, reading results
back as float64, running the oracle on the same storage arrays, and the tolerance rule."""
import numpy as np
import torch

import oracle
from paper_2506_01206_amd import synth

DEV = "cuda:0"

# Tolerances on outputs and states relative to the fp64 oracle: 1e-4 for float32 I/O, 2e-2 for
# bfloat16 I/O (one rounding of the output to 8 significant bits is 2^-9 ~ 2e-3 of that).
TOL = {synth.F32: 1e-4, synth.BF16: 2e-2}


def to_dev(a, io=None):
    """numpy storage array -> device tensor.  uint16 arrays are bfloat16 bit patterns."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if not a.flags.writeable:                                     # a read-only view (a broadcast, a stored fixture): torch wants its own
        a = a.copy()
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_host(t):
    """device tensor -> numpy storage array (bfloat16 comes back as uint16 bit patterns)."""
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def values(a):
    """numpy storage array -> float64 values."""
    if a.dtype == np.uint16:
        return oracle.widen(a, bf16=True)
    return a.astype(np.float64)


def W(a):
    """oracle input from a storage array (exact widening); None passes through."""
    if a is None:
        return None
    return oracle.widen(a, bf16=(a.dtype == np.uint16))


def assert_close(got, ref, tol, what=""):
    """|got - ref| <= tol * max(|ref|, rms(ref)) for every element (ref from the oracle)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), what + ": non-finite values in the GPU result"
    rms = float(np.sqrt(np.mean(ref * ref)))
    scale = np.maximum(np.abs(ref), rms)
    if rms == 0.0:
        assert np.all(got == 0.0), what
        return 0.0
    err = np.abs(got - ref) / scale
    worst = float(err.max())
    if worst > tol:
        i = np.unravel_index(int(err.argmax()), err.shape)
        raise AssertionError("%s: max scaled error %.3e > %.1e at %s (got %r, ref %r, rms %.3e)"
                             % (what, worst, tol, i, got[i], ref[i], rms))
    return worst


def oracle_scan(c, channels=None, h0=None, **kw):
    """Oracle scan on a prefill case dict (optionally on a subset of channels)."""
    sl = (lambda a: a) if channels is None else (lambda a: a[..., channels])
    rows = (lambda a: a) if channels is None else (lambda a: a[channels])
    args = dict(
        x=W(sl(c["x"])), dt=W(sl(c["dt"])), A=W(rows(c["A"])), Bm=W(c["Bm"]), Cm=W(c["Cm"]),
        Dskip=W(rows(c["Dskip"])), z=W(sl(c["z"])), dt_bias=W(rows(c["dt_bias"])),
        h0=None if h0 is None else (h0 if channels is None else h0[:, channels]))
    args.update(kw)
    return oracle.scan_fwd(**args)


def dev_case(c, keys=("x", "z", "Bm", "Cm", "dt", "A", "Dskip", "dt_bias", "conv_w", "conv_bias")):
    return {k: to_dev(c[k]) for k in keys if k in c}
