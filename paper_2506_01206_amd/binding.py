"""ctypes binding of libmamba_hip.so (the C ABI in include/mamba_hip.h).

Argument marshalling only: shapes and dtypes are read off the tensors, output
tensors are allocated with torch when the caller passes none, pointers and the
current HIP stream are handed to the C function, and a non-zero status raises.
Every step of the computation runs in the library's kernels.  There is no
fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# MAMBA_HIP_LIB names another build of the same library (the host-sanitizer run loads an instrumented one)
LIB_PATH = os.environ.get("MAMBA_HIP_LIB") or os.path.join(_HERE, "libmamba_hip.so")

MAMBA_F32 = 0
MAMBA_BF16 = 1
STATUS = dict(OK=0, NULL_POINTER=-1, BAD_SHAPE=-2, UNSUPPORTED=-3, MISALIGNED=-4, WORKSPACE=-5,
              ALIAS=-6)

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libmamba_hip.so is missing: build it with `python -m paper_2506_01206_amd.build` "
        "(there is no CPU or PyTorch fallback for the kernels)")

_vp, _i64, _int, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t


MAMBA_MAX_DEPTH = 16


class TreePlan(ctypes.Structure):
    """mamba_tree_plan_t of include/mamba_hip.h."""
    _n = MAMBA_MAX_DEPTH + 1
    _fields_ = [("gamma", ctypes.c_int32), ("n_caches", ctypes.c_int32),
                ("batch", ctypes.c_int64 * _n), ("cache_of_depth", ctypes.c_int32 * _n),
                ("parent_offset", ctypes.c_int64 * _n), ("cache_batch", ctypes.c_int64 * _n),
                ("conv_offset", ctypes.c_int64 * _n), ("ssm_offset", ctypes.c_int64 * _n),
                ("total_bytes", ctypes.c_int64)]


class BlockParams(ctypes.Structure):
    """mamba_block_params_t of include/mamba_hip.h."""
    _fields_ = [("d_model", ctypes.c_int64), ("d_inner", ctypes.c_int64), ("d_state", ctypes.c_int64),
                ("dt_rank", ctypes.c_int64), ("d_conv", ctypes.c_int32), ("eps", ctypes.c_float),
                ("norm_w", ctypes.c_void_p), ("in_proj_w", ctypes.c_void_p), ("conv_w", ctypes.c_void_p),
                ("conv_b", ctypes.c_void_p), ("x_proj_w", ctypes.c_void_p), ("dt_proj_w", ctypes.c_void_p),
                ("dt_bias", ctypes.c_void_p), ("A", ctypes.c_void_p), ("Dskip", ctypes.c_void_p),
                ("out_proj_w", ctypes.c_void_p)]


def _declare(lib):
    """Attach the C signatures of include/mamba_hip.h to a loaded library."""
    _bpp = ctypes.POINTER(BlockParams)
    lib.mamba_block_workspace_bytes.argtypes = [_bpp, _i64, _i64]
    lib.mamba_block_workspace_bytes.restype = _sz
    lib.mamba_block_workspace_layout.argtypes = [_bpp, _i64, _i64, ctypes.POINTER(ctypes.c_int64)]
    lib.mamba_block_workspace_layout.restype = _int
    lib.mamba_block_fwd.argtypes = [_bpp] + [_vp] * 7 + [_sz, _i64, _i64, _vp]
    lib.mamba_block_fwd.restype = _int
    lib.mamba_block_step.argtypes = [_bpp] + [_vp] * 8 + [_sz, _i64, _i64, _vp]
    lib.mamba_block_step.restype = _int
    lib.mamba2_ssd_workspace_bytes.argtypes = [_i64] * 5
    lib.mamba2_ssd_workspace_bytes.restype = _sz
    lib.mamba2_ssd_fwd.argtypes = [_vp] * 12 + [_sz] + [_i64] * 5 + [_int, _int, _vp]
    lib.mamba2_ssd_fwd.restype = _int
    lib.mamba2_state_step.argtypes = [_vp] * 12 + [_i64] * 5 + [_int, _int, _vp]
    lib.mamba2_state_step.restype = _int
    lib.mamba_embedding_fwd.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _int, _vp]
    lib.mamba_embedding_fwd.restype = _int
    lib.mamba_topk_fwd.argtypes = [_vp, _vp, _vp, _i64, _i64, _int, _int, _vp]
    lib.mamba_topk_fwd.restype = _int
    lib.mamba_tree_plan.argtypes = [ctypes.POINTER(ctypes.c_int32), _int, _i64, _i64, _i64, _int, _int,
                                    ctypes.POINTER(TreePlan)]
    lib.mamba_tree_plan.restype = _int
    lib.mamba_tree_parents.argtypes = [_vp, ctypes.POINTER(TreePlan), ctypes.POINTER(ctypes.c_int32), _vp]
    lib.mamba_tree_parents.restype = _int
    lib.mamba_linear_fwd.argtypes = [_vp] * 5 + [_i64, _vp, _i64, _vp, _i64, _i64, _i64, _int, _vp]
    lib.mamba_linear_fwd.restype = _int
    lib.mamba_rmsnorm_fwd.argtypes = [_vp, _vp, _vp, _i64, _i64, ctypes.c_float, _int, _vp]
    lib.mamba_rmsnorm_fwd.restype = _int
    lib.mamba_status_string.argtypes = [_int]
    lib.mamba_status_string.restype = ctypes.c_char_p
    lib.mamba_conv1d_fwd.argtypes = [_vp] * 6 + [_i64, _i64, _i64, _int, _int, _int, _vp]
    lib.mamba_conv1d_fwd.restype = _int
    lib.mamba_scan_workspace_bytes.argtypes = [_i64] * 5
    lib.mamba_scan_workspace_bytes.restype = _sz
    lib.mamba_scan_kernel.argtypes = [_i64] * 5
    lib.mamba_scan_kernel.restype = ctypes.c_char_p
    lib.mamba_scan_fwd.argtypes = [_vp] * 12 + [_sz] + [_i64] * 5 + [_int, _int, _vp]
    lib.mamba_scan_fwd.restype = _int
    lib.mamba_scan_fwd_static.argtypes = [_vp] * 11 + [_i64] * 5 + [_int, _int, _vp]
    lib.mamba_scan_fwd_static.restype = _int
    lib.mamba_conv1d_fwd_strided.argtypes = [_vp] * 8 + [_i64, _i64, _i64, _int, _int, _int, _vp]
    lib.mamba_conv1d_fwd_strided.restype = _int
    lib.mamba_scan_fwd_strided.argtypes = [_vp] * 16 + [_sz] + [_i64] * 4 + [_int, _int, _vp]
    lib.mamba_scan_fwd_strided.restype = _int
    lib.mamba_state_step.argtypes = [_vp] * 12 + [_i64] * 4 + [_int, _int, _vp]
    lib.mamba_state_step.restype = _int
    lib.mamba_state_fork.argtypes = [_vp] * 5 + [_i64] * 5 + [_int, _int, _vp]
    lib.mamba_state_fork.restype = _int
    lib.mamba_conv_state_step.argtypes = [_vp] * 17 + [_i64] * 4 + [_int] * 4 + [_vp]
    lib.mamba_conv_state_step.restype = _int
    return lib


lib = _declare(ctypes.CDLL(LIB_PATH))

EXPORTS = ("mamba_status_string", "mamba_conv1d_fwd", "mamba_scan_workspace_bytes", "mamba_scan_kernel",
           "mamba_scan_fwd", "mamba_scan_fwd_static", "mamba_conv1d_fwd_strided", "mamba_scan_fwd_strided", "mamba_state_step", "mamba_conv_state_step", "mamba_state_fork", "mamba_tree_plan",
           "mamba_tree_parents", "mamba_linear_fwd", "mamba_rmsnorm_fwd", "mamba_block_workspace_bytes",
           "mamba_block_workspace_layout", "mamba_block_fwd", "mamba_block_step", "mamba_embedding_fwd", "mamba_topk_fwd",
           "mamba2_ssd_workspace_bytes", "mamba2_ssd_fwd", "mamba2_state_step")


class MambaError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__("%s failed with status %d: %s" % (fn, status, mamba_status_string(status)))


def mamba_status_string(status: int) -> str:
    return lib.mamba_status_string(int(status)).decode()


def _check(fn, status):
    if status != 0:
        raise MambaError(fn, status)


def _io_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MAMBA_F32
    if t.dtype == torch.bfloat16:
        return MAMBA_BF16
    raise TypeError("I/O tensors must be float32 or bfloat16, got %s" % t.dtype)


def _ptr(t, dtype=None, shape=None, name="tensor"):
    """Device pointer of a contiguous CUDA tensor (None -> NULL), with dtype/shape checks."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return t.data_ptr() if t.numel() > 0 else None


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _scratch(nbytes, device, stream):
    """A workspace the binding allocates for one call and drops on return.  The caching allocator may hand the
    block to later work on the current stream, so when the call runs on another stream the block is tied to it."""
    ws = torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)
    if stream is not None and stream != torch.cuda.current_stream(device):
        ws.record_stream(stream)
    return ws


def mamba_conv1d_fwd(x, w, bias=None, conv_state_in=None, y=None, conv_state_out=None,
                     apply_silu=True, want_state=True, stream=None):
    """x (B,L,D) f32|bf16, w (D,K) f32 -> y (B,L,D), conv_state_out (B,D,K-1)."""
    B, L, D = x.shape
    K = w.shape[1]
    io = _io_code(x)
    if y is None:
        y = torch.empty_like(x)
    if conv_state_out is None and want_state:
        conv_state_out = torch.empty((B, D, K - 1), dtype=x.dtype, device=x.device)
    st = lib.mamba_conv1d_fwd(
        _ptr(x, name="x"), _ptr(w, torch.float32, (D, K), "w"), _ptr(bias, torch.float32, (D,), "bias"),
        _ptr(conv_state_in, x.dtype, (B, D, K - 1), "conv_state_in"), _ptr(y, x.dtype, (B, L, D), "y"),
        _ptr(conv_state_out, x.dtype, (B, D, K - 1), "conv_state_out"),
        B, L, D, K, int(bool(apply_silu)), io, _stream(stream))
    _check("mamba_conv1d_fwd", st)
    return y, conv_state_out


def mamba_scan_workspace_bytes(batch, L, D, N, chunk_len=0) -> int:
    return int(lib.mamba_scan_workspace_bytes(batch, L, D, N, chunk_len))


def mamba_scan_kernel(batch, L, D, N, chunk_len=0) -> str:
    """Name of the kernel family mamba_scan_fwd runs for this shape: chunked, direct, lanes or single."""
    return lib.mamba_scan_kernel(batch, L, D, N, chunk_len).decode()


def mamba_scan_fwd(x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, h0=None, out=None,
                   h_final=None, workspace=None, chunk_len=0, dt_softplus=True, want_state=True,
                   stream=None):
    """x, dt, z (B,L,D); Bm, Cm (B,L,N); A (D,N) f32 -> out (B,L,D), h_final (B,D,N) f32."""
    B, L, D = x.shape
    N = A.shape[1]
    io = _io_code(x)
    if out is None:
        out = torch.empty_like(x)
    if h_final is None and want_state:
        h_final = torch.empty((B, D, N), dtype=torch.float32, device=x.device)
    need = mamba_scan_workspace_bytes(B, L, D, N, chunk_len)
    if workspace is None and need > 0:
        workspace = _scratch(need, x.device, stream)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.mamba_scan_fwd(
        _ptr(x, name="x"), _ptr(dt, x.dtype, (B, L, D), "dt"), _ptr(A, torch.float32, (D, N), "A"),
        _ptr(Bm, x.dtype, (B, L, N), "Bm"), _ptr(Cm, x.dtype, (B, L, N), "Cm"),
        _ptr(Dskip, torch.float32, (D,), "Dskip"), _ptr(z, x.dtype, (B, L, D), "z"),
        _ptr(dt_bias, torch.float32, (D,), "dt_bias"), _ptr(h0, torch.float32, (B, D, N), "h0"),
        _ptr(out, x.dtype, (B, L, D), "out"), _ptr(h_final, torch.float32, (B, D, N), "h_final"),
        _ptr(workspace, name="workspace"), ws_bytes, B, L, D, N, int(chunk_len),
        int(bool(dt_softplus)), io, _stream(stream))
    _check("mamba_scan_fwd", st)
    return out, h_final


MAMBA_SCAN_STATIC_BYTES = 32 << 20


def mamba_scan_fwd_static(x, dt, A, Bm, Cm, Dskip, z, dt_bias, h0, out, h_final, chunk_len=0, dt_softplus=True,
                          stream=None):
    """mamba_scan_fwd with the chunk states in the library's own device buffer.  Allocates nothing: the caller
    passes every tensor, ``out`` (B,L,D) and ``h_final`` (B,D,N) or None included."""
    B, L, D = x.shape
    N = A.shape[1]
    st = lib.mamba_scan_fwd_static(
        _ptr(x, name="x"), _ptr(dt, x.dtype, (B, L, D), "dt"), _ptr(A, torch.float32, (D, N), "A"),
        _ptr(Bm, x.dtype, (B, L, N), "Bm"), _ptr(Cm, x.dtype, (B, L, N), "Cm"),
        _ptr(Dskip, torch.float32, (D,), "Dskip"), _ptr(z, x.dtype, (B, L, D), "z"),
        _ptr(dt_bias, torch.float32, (D,), "dt_bias"), _ptr(h0, torch.float32, (B, D, N), "h0"),
        _ptr(out, x.dtype, (B, L, D), "out"), _ptr(h_final, torch.float32, (B, D, N), "h_final"),
        B, L, D, N, int(chunk_len), int(bool(dt_softplus)), _io_code(x), _stream(stream))
    _check("mamba_scan_fwd_static", st)
    return out, h_final


def _view(t, dtype=None, shape=None, name="tensor"):
    """(device pointer, host stride triple) of a CUDA tensor of logical shape (B, L, D) in any layout."""
    if t is None:
        return None, None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return (t.data_ptr() if t.numel() > 0 else None), (ctypes.c_int64 * 3)(*t.stride())


def mamba_conv1d_fwd_strided(x, w, bias=None, conv_state_in=None, y=None, conv_state_out=None,
                             apply_silu=True, want_state=True, stream=None):
    """mamba_conv1d_fwd for x and y of logical shape (B,L,D) in any layout (a transposed (B,D,L) tensor, a column
    range of a wider tensor): their strides go to the library as they are.  y defaults to a contiguous tensor."""
    B, L, D = x.shape
    K = w.shape[1]
    if y is None:
        y = torch.empty((B, L, D), dtype=x.dtype, device=x.device)
    if conv_state_out is None and want_state:
        conv_state_out = torch.empty((B, D, K - 1), dtype=x.dtype, device=x.device)
    xp, xs = _view(x, name="x")
    yp, ys = _view(y, x.dtype, (B, L, D), "y")
    st = lib.mamba_conv1d_fwd_strided(
        xp, xs, _ptr(w, torch.float32, (D, K), "w"), _ptr(bias, torch.float32, (D,), "bias"),
        _ptr(conv_state_in, x.dtype, (B, D, K - 1), "conv_state_in"), yp, ys,
        _ptr(conv_state_out, x.dtype, (B, D, K - 1), "conv_state_out"),
        B, L, D, K, int(bool(apply_silu)), _io_code(x), _stream(stream))
    _check("mamba_conv1d_fwd_strided", st)
    return y, conv_state_out


def mamba_scan_fwd_strided(x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, h0=None, out=None,
                           h_final=None, workspace=None, dt_softplus=True, want_state=True, stream=None):
    """mamba_scan_fwd for x, dt, z, out of logical shape (B,L,D) in any layout, each with its own strides;
    Bm, Cm (B,L,N) and the rest contiguous as there.  out defaults to a contiguous tensor."""
    B, L, D = x.shape
    N = A.shape[1]
    if out is None:
        out = torch.empty((B, L, D), dtype=x.dtype, device=x.device)
    if h_final is None and want_state:
        h_final = torch.empty((B, D, N), dtype=torch.float32, device=x.device)
    need = mamba_scan_workspace_bytes(B, L, D, N, 0)     # only used when every layout is the contiguous one
    if workspace is None and need > 0:
        workspace = _scratch(need, x.device, stream)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    xp, xs = _view(x, name="x")
    dp, ds = _view(dt, x.dtype, (B, L, D), "dt")
    zp, zs = _view(z, x.dtype, (B, L, D), "z")
    op, os_ = _view(out, x.dtype, (B, L, D), "out")
    st = lib.mamba_scan_fwd_strided(
        xp, xs, dp, ds, _ptr(A, torch.float32, (D, N), "A"), _ptr(Bm, x.dtype, (B, L, N), "Bm"),
        _ptr(Cm, x.dtype, (B, L, N), "Cm"), _ptr(Dskip, torch.float32, (D,), "Dskip"), zp, zs,
        _ptr(dt_bias, torch.float32, (D,), "dt_bias"), _ptr(h0, torch.float32, (B, D, N), "h0"), op, os_,
        _ptr(h_final, torch.float32, (B, D, N), "h_final"), _ptr(workspace, name="workspace"), ws_bytes,
        B, L, D, N, int(bool(dt_softplus)), _io_code(x), _stream(stream))
    _check("mamba_scan_fwd_strided", st)
    return out, h_final


def mamba_state_step(h_in, x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, parent_idx=None,
                     h_out=None, out=None, dt_softplus=True, stream=None):
    """h_in (n_in,D,N) f32; x, dt, z (n_out,D); Bm, Cm (n_out,N); parent_idx int32[n_out]
    -> h_out (n_out,D,N), out (n_out,D).  Pass h_out=h_in for the in-place sequential step."""
    n_in, D, N = h_in.shape
    n_out = x.shape[0]
    io = _io_code(x)
    if h_out is None:
        h_out = torch.empty((n_out, D, N), dtype=torch.float32, device=x.device)
    if out is None:
        out = torch.empty_like(x)
    st = lib.mamba_state_step(
        _ptr(h_out, torch.float32, (n_out, D, N), "h_out"), _ptr(h_in, torch.float32, name="h_in"),
        _ptr(parent_idx, torch.int32, (n_out,), "parent_idx"), _ptr(x, name="x"),
        _ptr(dt, x.dtype, (n_out, D), "dt"), _ptr(A, torch.float32, (D, N), "A"),
        _ptr(Bm, x.dtype, (n_out, N), "Bm"), _ptr(Cm, x.dtype, (n_out, N), "Cm"),
        _ptr(Dskip, torch.float32, (D,), "Dskip"), _ptr(z, x.dtype, (n_out, D), "z"),
        _ptr(dt_bias, torch.float32, (D,), "dt_bias"), _ptr(out, x.dtype, (n_out, D), "out"),
        n_out, n_in, D, N, int(bool(dt_softplus)), io, _stream(stream))
    _check("mamba_state_step", st)
    return h_out, out


def mamba_conv_state_step(h_in, conv_state_in, x, conv_w, conv_bias, dt, A, Bm, Cm, Dskip=None, z=None,
                          dt_bias=None, parent_idx=None, h_out=None, conv_state_out=None, out=None, xc_out=None,
                          want_xc=False, apply_silu=True, dt_softplus=True, stream=None):
    """Fork + conv step + state update of one layer in one launch.  h_in (n_in,D,N) f32, conv_state_in
    (n_in,D,K-1), x (n_out,D) the input before the conv, conv_w (D,K) f32; the rest as mamba_state_step.
    -> h_out, conv_state_out (n_out,D,K-1), out (n_out,D), x_c (n_out,D) or None."""
    n_in, D, N = h_in.shape
    n_out = x.shape[0]
    K = conv_w.shape[1]
    io = _io_code(x)
    if h_out is None:
        h_out = torch.empty((n_out, D, N), dtype=torch.float32, device=x.device)
    if conv_state_out is None:
        conv_state_out = torch.empty((n_out, D, K - 1), dtype=x.dtype, device=x.device)
    if out is None:
        out = torch.empty_like(x)
    if xc_out is None and want_xc:
        xc_out = torch.empty_like(x)
    st = lib.mamba_conv_state_step(
        _ptr(h_out, torch.float32, (n_out, D, N), "h_out"), _ptr(h_in, torch.float32, name="h_in"),
        _ptr(conv_state_out, x.dtype, (n_out, D, K - 1), "conv_state_out"),
        _ptr(conv_state_in, x.dtype, (n_in, D, K - 1), "conv_state_in"),
        _ptr(parent_idx, torch.int32, (n_out,), "parent_idx"), _ptr(x, name="x"),
        _ptr(conv_w, torch.float32, (D, K), "conv_w"), _ptr(conv_bias, torch.float32, (D,), "conv_bias"),
        _ptr(dt, x.dtype, (n_out, D), "dt"), _ptr(A, torch.float32, (D, N), "A"),
        _ptr(Bm, x.dtype, (n_out, N), "Bm"), _ptr(Cm, x.dtype, (n_out, N), "Cm"),
        _ptr(Dskip, torch.float32, (D,), "Dskip"), _ptr(z, x.dtype, (n_out, D), "z"),
        _ptr(dt_bias, torch.float32, (D,), "dt_bias"), _ptr(out, x.dtype, (n_out, D), "out"),
        _ptr(xc_out, x.dtype, (n_out, D), "xc_out"),
        n_out, n_in, D, N, K, int(bool(apply_silu)), int(bool(dt_softplus)), io, _stream(stream))
    _check("mamba_conv_state_step", st)
    return h_out, conv_state_out, out, xc_out


def mamba_state_fork(conv_src, ssm_src, parent_idx, conv_dst=None, ssm_dst=None, stream=None):
    """conv_src (n_layers,n_in,D,K-1) f32|bf16 or None, ssm_src (n_layers,n_in,D,N) f32 or None,
    parent_idx int32[n_out] -> gathered copies (n_layers,n_out,...)."""
    ref = conv_src if conv_src is not None else ssm_src
    n_layers, n_in, D = ref.shape[0], ref.shape[1], ref.shape[2]
    n_out = parent_idx.shape[0]
    K, N, cd = 1, 0, MAMBA_F32
    if conv_src is not None:
        K = conv_src.shape[3] + 1
        cd = _io_code(conv_src)
        if conv_dst is None:
            conv_dst = torch.empty((n_layers, n_out, D, K - 1), dtype=conv_src.dtype, device=ref.device)
    if ssm_src is not None:
        N = ssm_src.shape[3]
        if ssm_dst is None:
            ssm_dst = torch.empty((n_layers, n_out, D, N), dtype=torch.float32, device=ref.device)
    st = lib.mamba_state_fork(
        _ptr(conv_dst, name="conv_dst"), _ptr(conv_src, name="conv_src"),
        _ptr(ssm_dst, torch.float32, name="ssm_dst"), _ptr(ssm_src, torch.float32, name="ssm_src"),
        _ptr(parent_idx, torch.int32, name="parent_idx"), n_layers, n_out, n_in, D, N, K, cd,
        _stream(stream))
    _check("mamba_state_fork", st)
    return conv_dst, ssm_dst


def _tree_array(tree):
    return (ctypes.c_int32 * len(tree))(*[int(n) for n in tree])


def mamba_tree_plan(tree, n_layers, D, N, K, conv_dtype=torch.bfloat16) -> TreePlan:
    """Batch sizes and cache layout for a tree configuration (N_1..N_gamma); host arithmetic only."""
    plan = TreePlan()
    code = MAMBA_F32 if conv_dtype == torch.float32 else MAMBA_BF16 if conv_dtype == torch.bfloat16 else -1
    st = lib.mamba_tree_plan(_tree_array(tree), len(tree), n_layers, D, N, K, code, ctypes.byref(plan))
    _check("mamba_tree_plan", st)
    return plan


def mamba_tree_parents(slab, plan: TreePlan, tree, stream=None):
    """Write the parent-index arrays of every branching draft position into the slab."""
    st = lib.mamba_tree_parents(_ptr(slab, torch.uint8, name="slab"), ctypes.byref(plan), _tree_array(tree),
                                _stream(stream))
    _check("mamba_tree_parents", st)


def mamba_linear_fwd(x, w, bias=None, residual=None, splits=None, outs=None, stream=None):
    """x (M,K) bf16, w (N,K) bf16 -> x @ w.T (+ bias) (+ residual).  ``splits`` = widths of up to three
    output tensors that share the N columns (default: one tensor of width N); returns a tuple."""
    M, K = x.shape
    N = w.shape[0]
    widths = [N] if splits is None else list(splits)
    assert sum(widths) == N and 1 <= len(widths) <= 3
    if outs is None:
        outs = [torch.empty((M, n), dtype=x.dtype, device=x.device) for n in widths]
    widths += [0] * (3 - len(widths))
    outs = list(outs) + [None] * (3 - len(outs))
    st = lib.mamba_linear_fwd(
        _ptr(x, name="x"), _ptr(w, x.dtype, (N, K), "w"), _ptr(bias, torch.float32, (N,), "bias"),
        _ptr(residual, x.dtype, (M, N), "residual"),
        _ptr(outs[0], x.dtype, (M, widths[0]), "out0"), widths[0],
        _ptr(outs[1], x.dtype, (M, widths[1]), "out1"), widths[1],
        _ptr(outs[2], x.dtype, (M, widths[2]), "out2"), widths[2], M, K, _io_code(x), _stream(stream))
    _check("mamba_linear_fwd", st)
    return tuple(o for o in outs if o is not None)


def mamba_rmsnorm_fwd(x, w, eps=1e-5, y=None, stream=None):
    """x (M,C) bf16, w (C) f32 -> x * rsqrt(mean(x^2) + eps) * w."""
    M, C = x.shape
    if y is None:
        y = torch.empty_like(x)
    st = lib.mamba_rmsnorm_fwd(_ptr(x, name="x"), _ptr(w, torch.float32, (C,), "w"), _ptr(y, x.dtype, (M, C), "y"),
                               M, C, float(eps), _io_code(x), _stream(stream))
    _check("mamba_rmsnorm_fwd", st)
    return y


class Block:
    """Parameters of one Mamba block on the device (a mamba_block_params_t plus the tensors it points
    to, kept alive).  ``w`` maps names to device tensors: norm_w (d_model) f32, in_proj_w (2 d_inner,
    d_model) bf16, conv_w (d_inner, d_conv) f32, conv_b (d_inner) f32 or None, x_proj_w (dt_rank + 2
    d_state, d_inner) bf16, dt_proj_w (d_inner, dt_rank) bf16, dt_bias, Dskip (d_inner) f32, A (d_inner,
    d_state) f32, out_proj_w (d_model, d_inner) bf16."""

    def __init__(self, w, eps=1e-5):
        self.w = dict(w)
        d_inner, d_conv = w["conv_w"].shape
        d_model = w["norm_w"].shape[0]
        d_state = w["A"].shape[1]
        dt_rank = w["dt_proj_w"].shape[1]
        f32, bf = torch.float32, torch.bfloat16
        self.c = BlockParams(
            d_model, d_inner, d_state, dt_rank, d_conv, float(eps),
            _ptr(w["norm_w"], f32, (d_model,), "norm_w"), _ptr(w["in_proj_w"], bf, (2 * d_inner, d_model), "in_proj_w"),
            _ptr(w["conv_w"], f32, name="conv_w"), _ptr(w.get("conv_b"), f32, (d_inner,), "conv_b"),
            _ptr(w["x_proj_w"], bf, (dt_rank + 2 * d_state, d_inner), "x_proj_w"),
            _ptr(w["dt_proj_w"], bf, (d_inner, dt_rank), "dt_proj_w"), _ptr(w["dt_bias"], f32, (d_inner,), "dt_bias"),
            _ptr(w["A"], f32, (d_inner, d_state), "A"), _ptr(w["Dskip"], f32, (d_inner,), "Dskip"),
            _ptr(w["out_proj_w"], bf, (d_model, d_inner), "out_proj_w"))
        self.d_model, self.d_inner, self.d_state, self.dt_rank, self.d_conv = d_model, d_inner, d_state, dt_rank, d_conv


def mamba_block_workspace_bytes(block: Block, batch, L) -> int:
    return int(lib.mamba_block_workspace_bytes(ctypes.byref(block.c), batch, L))


def mamba_block_workspace_layout(block: Block, batch, L, workspace):
    """Views of the stage tensors mamba_block_fwd left in ``workspace`` (uint8 device tensor) on its last call with
    this batch and L: dict with dt, z, x_c, y (rows, d_inner), dt_low (rows, dt_rank), B, C (rows, d_state), bf16."""
    off = (ctypes.c_int64 * 7)()
    _check("mamba_block_workspace_layout", lib.mamba_block_workspace_layout(ctypes.byref(block.c), batch, L, off))
    rows = batch * L
    widths = dict(dt=block.d_inner, z=block.d_inner, x_c=block.d_inner, y=block.d_inner, dt_low=block.dt_rank,
                  B=block.d_state, C=block.d_state)
    return {k: workspace[off[i]:off[i] + rows * w * 2].view(torch.bfloat16).view(rows, w)
            for i, (k, w) in enumerate(widths.items())}


def mamba_block_fwd(block: Block, hidden, hidden_out=None, conv_state_in=None, h0=None, conv_state_out=None,
                    h_final=None, workspace=None, want_state=True, stream=None):
    """hidden (B,L,d_model) bf16 -> hidden + mixer(rmsnorm(hidden)); also the conv and SSM states."""
    B, L, dm = hidden.shape
    D, N, K = block.d_inner, block.d_state, block.d_conv
    if hidden_out is None:
        hidden_out = torch.empty_like(hidden)
    if want_state and conv_state_out is None:
        conv_state_out = torch.empty((B, D, K - 1), dtype=hidden.dtype, device=hidden.device)
    if want_state and h_final is None:
        h_final = torch.empty((B, D, N), dtype=torch.float32, device=hidden.device)
    need = mamba_block_workspace_bytes(block, B, L)
    if workspace is None:
        workspace = _scratch(need, hidden.device, stream)
    st = lib.mamba_block_fwd(
        ctypes.byref(block.c), _ptr(hidden, torch.bfloat16, name="hidden"),
        _ptr(hidden_out, torch.bfloat16, (B, L, dm), "hidden_out"),
        _ptr(conv_state_in, torch.bfloat16, (B, D, K - 1), "conv_state_in"),
        _ptr(conv_state_out, torch.bfloat16, (B, D, K - 1), "conv_state_out"),
        _ptr(h0, torch.float32, (B, D, N), "h0"), _ptr(h_final, torch.float32, (B, D, N), "h_final"),
        _ptr(workspace, name="workspace"), workspace.numel() * workspace.element_size(), B, L, _stream(stream))
    _check("mamba_block_fwd", st)
    return hidden_out, conv_state_out, h_final


def mamba_block_step(block: Block, hidden, conv_src, ssm_src, parent_idx=None, conv_dst=None, ssm_dst=None,
                     hidden_out=None, workspace=None, stream=None):
    """One token for n_out draft branches: hidden (n_out,d_model); states (n_in,D,K-1) / (n_in,D,N).
    With parent_idx the children's states go to conv_dst / ssm_dst; without, the step is in place."""
    n_out, dm = hidden.shape
    n_in = conv_src.shape[0]
    D, N, K = block.d_inner, block.d_state, block.d_conv
    if hidden_out is None:
        hidden_out = torch.empty_like(hidden)
    if parent_idx is None:
        conv_dst, ssm_dst = conv_src, ssm_src
    else:
        if conv_dst is None:
            conv_dst = torch.empty((n_out, D, K - 1), dtype=conv_src.dtype, device=hidden.device)
        if ssm_dst is None:
            ssm_dst = torch.empty((n_out, D, N), dtype=torch.float32, device=hidden.device)
    need = mamba_block_workspace_bytes(block, n_out, 1)
    if workspace is None:
        workspace = _scratch(need, hidden.device, stream)
    st = lib.mamba_block_step(
        ctypes.byref(block.c), _ptr(hidden, torch.bfloat16, name="hidden"),
        _ptr(hidden_out, torch.bfloat16, (n_out, dm), "hidden_out"),
        _ptr(conv_src, torch.bfloat16, (n_in, D, K - 1), "conv_src"), _ptr(conv_dst, torch.bfloat16, (n_out, D, K - 1), "conv_dst"),
        _ptr(ssm_src, torch.float32, (n_in, D, N), "ssm_src"), _ptr(ssm_dst, torch.float32, (n_out, D, N), "ssm_dst"),
        _ptr(parent_idx, torch.int32, (n_out,), "parent_idx"), _ptr(workspace, name="workspace"),
        workspace.numel() * workspace.element_size(), n_out, n_in, _stream(stream))
    _check("mamba_block_step", st)
    return hidden_out, conv_dst, ssm_dst


def mamba_embedding_fwd(tokens, table, out=None, stream=None):
    """tokens int32[M], table (V,dm) bf16 -> (M,dm) rows."""
    M = tokens.shape[0]
    V, dm = table.shape
    if out is None:
        out = torch.empty((M, dm), dtype=table.dtype, device=table.device)
    st = lib.mamba_embedding_fwd(_ptr(tokens, torch.int32, (M,), "tokens"), _ptr(table, name="table"),
                                 _ptr(out, table.dtype, (M, dm), "out"), M, V, dm, _io_code(table), _stream(stream))
    _check("mamba_embedding_fwd", st)
    return out


def mamba_topk_fwd(logits, k, idx=None, val=None, stream=None):
    """logits (M,V) bf16 -> idx int32 (M,k), val float32 (M,k), largest first, ties to the lower index."""
    M, V = logits.shape
    if idx is None:
        idx = torch.empty((M, k), dtype=torch.int32, device=logits.device)
    if val is None:
        val = torch.empty((M, k), dtype=torch.float32, device=logits.device)
    st = lib.mamba_topk_fwd(_ptr(logits, name="logits"), _ptr(idx, torch.int32, (M, k), "idx"),
                            _ptr(val, torch.float32, (M, k), "val"), M, V, int(k), _io_code(logits), _stream(stream))
    _check("mamba_topk_fwd", st)
    return idx, val


def mamba2_ssd_workspace_bytes(batch, L, H, P, N) -> int:
    return int(lib.mamba2_ssd_workspace_bytes(batch, L, H, P, N))


def mamba2_ssd_fwd(x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, h0=None, out=None, h_final=None,
                   workspace=None, want_state=True, dt_softplus=True, stream=None):
    """Scalar-decay layer core: x, z (B,L,H,P) bf16; dt (B,L,H); Bm, Cm (B,L,N); A, Dskip, dt_bias (H) f32;
    h0 (B,H,P,N) f32 -> out (B,L,H,P), h_final (B,H,P,N)."""
    B, L, H, P = x.shape
    N = Bm.shape[-1]
    if out is None:
        out = torch.empty_like(x)
    if want_state and h_final is None:
        h_final = torch.empty((B, H, P, N), dtype=torch.float32, device=x.device)
    need = mamba2_ssd_workspace_bytes(B, L, H, P, N)
    if workspace is None:
        workspace = _scratch(need, x.device, stream)
    st = lib.mamba2_ssd_fwd(
        _ptr(x, name="x"), _ptr(dt, x.dtype, (B, L, H), "dt"), _ptr(A, torch.float32, (H,), "A"),
        _ptr(Bm, x.dtype, (B, L, N), "Bm"), _ptr(Cm, x.dtype, (B, L, N), "Cm"), _ptr(Dskip, torch.float32, (H,), "Dskip"),
        _ptr(z, x.dtype, (B, L, H, P), "z"), _ptr(dt_bias, torch.float32, (H,), "dt_bias"),
        _ptr(h0, torch.float32, (B, H, P, N), "h0"), _ptr(out, x.dtype, (B, L, H, P), "out"),
        _ptr(h_final, torch.float32, (B, H, P, N), "h_final"), _ptr(workspace, name="workspace"),
        workspace.numel() * workspace.element_size(), B, L, H, P, N, int(bool(dt_softplus)), _io_code(x), _stream(stream))
    _check("mamba2_ssd_fwd", st)
    return out, h_final


def mamba2_state_step(h_in, x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, parent_idx=None, h_out=None, out=None,
                      dt_softplus=True, stream=None):
    """h_in (n_in,H,P,N) f32; x, z (n_out,H,P); dt (n_out,H); Bm, Cm (n_out,N) -> h_out (n_out,H,P,N), out (n_out,H,P)."""
    n_in, H, P, N = h_in.shape
    n_out = x.shape[0]
    if h_out is None:
        h_out = torch.empty((n_out, H, P, N), dtype=torch.float32, device=x.device)
    if out is None:
        out = torch.empty_like(x)
    st = lib.mamba2_state_step(
        _ptr(h_out, torch.float32, (n_out, H, P, N), "h_out"), _ptr(h_in, torch.float32, name="h_in"),
        _ptr(parent_idx, torch.int32, (n_out,), "parent_idx"), _ptr(x, name="x"), _ptr(dt, x.dtype, (n_out, H), "dt"),
        _ptr(A, torch.float32, (H,), "A"), _ptr(Bm, x.dtype, (n_out, N), "Bm"), _ptr(Cm, x.dtype, (n_out, N), "Cm"),
        _ptr(Dskip, torch.float32, (H,), "Dskip"), _ptr(z, x.dtype, (n_out, H, P), "z"),
        _ptr(dt_bias, torch.float32, (H,), "dt_bias"), _ptr(out, x.dtype, (n_out, H, P), "out"),
        n_out, n_in, H, P, N, int(bool(dt_softplus)), _io_code(x), _stream(stream))
    _check("mamba2_state_step", st)
    return h_out, out
