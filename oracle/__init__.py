"""fp64 CPU oracle for the selective-SSM layer core (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It never imports the GPU package and shares nothing with it.

The arithmetic lives in mamba_oracle.c (plain loops, double precision); this
module compiles it with gcc on first use, widens inputs exactly to float64 and
marshals arguments.  Inputs may be float64/float32 numpy arrays, or uint16
arrays holding bfloat16 bit patterns (pass ``bf16=True`` to ``widen``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mamba_oracle.c")
_LIB = os.path.join(_HERE, "libmamba_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle into oracle/libmamba_oracle.so (gcc, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        other = os.environ.get("MAMBA_ORACLE_LIB")       # another build of mamba_oracle.c (the sanitizer run)
        if not other:
            build()
        lib = ctypes.CDLL(other or _LIB)
        dp = ctypes.c_void_p
        lg = ctypes.c_long
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        lib.oracle_conv1d_fwd.argtypes = [dp] * 6 + [lg, lg, lg, ctypes.c_int, ctypes.c_int]
        lib.oracle_conv1d_fwd.restype = None
        lib.oracle_scan_fwd.argtypes = [dp] * 11 + [lg, lg, lg, lg, ctypes.c_int]
        lib.oracle_scan_fwd.restype = None
        lib.oracle_state_step.argtypes = [dp] * 12 + [lg, lg, lg, lg, ctypes.c_int]
        lib.oracle_state_step.restype = None
        lib.oracle_state_fork.argtypes = [dp] * 5 + [lg] * 5
        lib.oracle_state_fork.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def widen(a, bf16: bool = False):
    """Exact conversion of an input array to contiguous float64.

    bf16=True: ``a`` is a uint16 array of bfloat16 bit patterns; a bfloat16 is
    the upper half of an IEEE float32, so widening is a 16-bit shift."""
    if a is None:
        return None
    a = np.asarray(a)
    if bf16:
        assert a.dtype == np.uint16, a.dtype
        f32 = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
        return np.ascontiguousarray(f32, dtype=np.float64)
    assert a.dtype in (np.float32, np.float64), a.dtype
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f64(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def conv1d_fwd(x, w, bias=None, conv_state_in=None, apply_silu=True, want_state=True):
    """x (B,L,D), w (D,K), bias (D), conv_state_in (B,D,K-1) -> y (B,L,D), conv_state_out."""
    x = _f64(x)
    B, L, D = x.shape
    w = _f64(w)
    K = w.shape[1]
    assert w.shape == (D, K) and K >= 1
    bias = _f64(bias, (D,))
    conv_state_in = _f64(conv_state_in, (B, D, K - 1))
    y = np.empty((B, L, D), dtype=np.float64)
    st = np.empty((B, D, K - 1), dtype=np.float64) if want_state else None
    _load().oracle_conv1d_fwd(_p(x), _p(w), _p(bias), _p(conv_state_in), _p(y), _p(st),
                              B, L, D, K, int(bool(apply_silu)))
    return y, st


def scan_fwd(x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, h0=None, dt_softplus=True):
    """x, dt, z (B,L,D); Bm, Cm (B,L,N); A (D,N); Dskip, dt_bias (D); h0 (B,D,N)
    -> out (B,L,D), h_final (B,D,N), all float64."""
    x = _f64(x)
    B, L, D = x.shape
    A = _f64(A)
    N = A.shape[1]
    assert A.shape == (D, N) and N <= 256
    dt = _f64(dt, (B, L, D))
    Bm = _f64(Bm, (B, L, N))
    Cm = _f64(Cm, (B, L, N))
    Dskip = _f64(Dskip, (D,))
    z = _f64(z, (B, L, D))
    dt_bias = _f64(dt_bias, (D,))
    h0 = _f64(h0, (B, D, N))
    out = np.empty((B, L, D), dtype=np.float64)
    hf = np.empty((B, D, N), dtype=np.float64)
    _load().oracle_scan_fwd(_p(x), _p(dt), _p(A), _p(Bm), _p(Cm), _p(Dskip), _p(z), _p(dt_bias),
                            _p(h0), _p(out), _p(hf), B, L, D, N, int(bool(dt_softplus)))
    return out, hf


def state_step(h_in, x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, parent=None,
               dt_softplus=True):
    """h_in (n_in,D,N); x, dt, z (n_out,D); Bm, Cm (n_out,N); parent int32[n_out] or None
    -> h_out (n_out,D,N), out (n_out,D)."""
    h_in = _f64(h_in)
    n_in, D, N = h_in.shape
    x = _f64(x)
    n_out = x.shape[0]
    assert x.shape == (n_out, D)
    if parent is None:
        assert n_in == n_out
    else:
        parent = np.ascontiguousarray(parent, dtype=np.int32)
        assert parent.shape == (n_out,)
        assert n_out == 0 or (parent.min() >= 0 and parent.max() < n_in)
    dt = _f64(dt, (n_out, D))
    A = _f64(A, (D, N))
    Bm = _f64(Bm, (n_out, N))
    Cm = _f64(Cm, (n_out, N))
    Dskip = _f64(Dskip, (D,))
    z = _f64(z, (n_out, D))
    dt_bias = _f64(dt_bias, (D,))
    h_out = np.empty((n_out, D, N), dtype=np.float64)
    out = np.empty((n_out, D), dtype=np.float64)
    _load().oracle_state_step(_p(h_out), _p(h_in), _p(parent), _p(x), _p(dt), _p(A), _p(Bm), _p(Cm),
                              _p(Dskip), _p(z), _p(dt_bias), _p(out), n_out, n_in, D, N,
                              int(bool(dt_softplus)))
    return h_out, out


def state_fork(conv_src, ssm_src, parent):
    """conv_src (n_layers,n_in,D,K-1) any dtype, ssm_src (n_layers,n_in,D,N) any dtype,
    parent int32[n_out] -> gathered copies (n_layers,n_out,...), byte-exact.  Either source
    may be None."""
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    n_out = parent.shape[0]
    ref = conv_src if conv_src is not None else ssm_src
    n_layers, n_in = ref.shape[0], ref.shape[1]
    assert n_out == 0 or (parent.min() >= 0 and parent.max() < n_in)
    outs = []
    rows = []
    for src in (conv_src, ssm_src):
        if src is None:
            outs.append(None)
            rows.append(0)
            continue
        src = np.ascontiguousarray(src)
        assert src.shape[0] == n_layers and src.shape[1] == n_in
        outs.append((src, np.empty((n_layers, n_out) + src.shape[2:], dtype=src.dtype)))
        rows.append(int(np.prod(src.shape[2:])) * src.dtype.itemsize)
    cs, cd = outs[0] if outs[0] is not None else (None, None)
    ss, sd = outs[1] if outs[1] is not None else (None, None)
    _load().oracle_state_fork(_p(cd), _p(cs), _p(sd), _p(ss), _p(parent),
                              n_layers, n_out, n_in, rows[0], rows[1])
    return cd, sd


# ---------------------------------------------------------------------------------------------
# Dense parts of the block (plain numpy, float64).  The Mamba-130M drafter of the paper (Sec. 3.1)
# wraps the selective SSM core in RMSNorm, in_proj, x_proj, dt_proj and out_proj with a residual.
def linear(x, w, bias=None, residual=None):
    """x (M,K), w (N,K) -> x @ w^T (+ bias) (+ residual), float64 (numpy.matmul is the contraction)."""
    out = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    if bias is not None:
        out = out + np.asarray(bias, dtype=np.float64)[None, :]
    if residual is not None:
        out = out + np.asarray(residual, dtype=np.float64)
    return out


def rmsnorm(x, w, eps):
    """y[m,:] = x[m,:] / sqrt(mean(x[m,:]^2) + eps) * w."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + float(eps)) * np.asarray(w, dtype=np.float64)


def _round_bf16(a):
    """float64 -> nearest bfloat16 value (ties to even), as float64: the rounding a tensor gets when a
    stage stores it in bf16."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return (((u + r) >> np.uint32(16)) << np.uint32(16)).view(np.float32).astype(np.float64)


def block_fwd(w, hidden, conv_state_in=None, h0=None, eps=1e-5, round_between=True):
    """One Mamba block on (B,L,d_model) float64 activations: rmsnorm, in_proj -> x | z, conv1d + silu,
    x_proj -> dt_low | B | C, dt_proj, selective scan gated by silu(z), out_proj, residual.
    round_between=True rounds every tensor that passes between two stages to bf16 (the storage
    type of the activations); False evaluates the block in float64 throughout.
    ``w``: norm_w, in_proj_w (2D,dm), conv_w, conv_b, x_proj_w (R+2N,D), dt_proj_w (D,R), dt_bias, A,
    Dskip, out_proj_w (dm,D), all float64 values.  Returns hidden_out, conv_state, ssm_state."""
    rb = _round_bf16 if round_between else (lambda a: np.asarray(a, dtype=np.float64))
    B, L, dm = hidden.shape
    D, N = w["A"].shape
    R = w["dt_proj_w"].shape[1]
    u = rb(rmsnorm(hidden.reshape(B * L, dm), w["norm_w"], eps))
    xz = rb(linear(u, w["in_proj_w"]))
    x, z = xz[:, :D].reshape(B, L, D), xz[:, D:].reshape(B, L, D)
    xc, conv_state = conv1d_fwd(x, w["conv_w"], w.get("conv_b"), conv_state_in, apply_silu=True)
    xc = rb(xc)
    proj = rb(linear(xc.reshape(B * L, D), w["x_proj_w"]))
    dtl, Bm, Cm = proj[:, :R], proj[:, R:R + N].reshape(B, L, N), proj[:, R + N:].reshape(B, L, N)
    dt = rb(linear(dtl, w["dt_proj_w"])).reshape(B, L, D)
    y, h_final = scan_fwd(xc, dt, w["A"], Bm, Cm, w["Dskip"], z, w["dt_bias"], h0)
    y = rb(y)
    out = linear(y.reshape(B * L, D), w["out_proj_w"], None, hidden.reshape(B * L, dm)).reshape(B, L, dm)
    return out, conv_state, h_final


def embedding(tokens, table):
    """Rows of the vocabulary table for each token (a gather)."""
    return np.asarray(table)[np.asarray(tokens, dtype=np.int64)]


def topk(logits, k):
    """Per row the k largest logits, largest first, equal values ordered by index (numpy.lexsort);
    NaN never wins.  Returns (idx int32 (M,k), val float64 (M,k)); missing entries are idx -1, val -inf."""
    x = np.array(logits, dtype=np.float64)
    x[np.isnan(x)] = -np.inf
    M, V = x.shape
    idx = np.full((M, k), -1, dtype=np.int32)
    val = np.full((M, k), -np.inf)
    for m in range(M):
        order = np.lexsort((np.arange(V), -x[m]))[:k]          # primary: value descending, then index
        idx[m, :order.size] = order
        val[m, :order.size] = x[m, order]
    return idx, val
