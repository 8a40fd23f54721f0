"""Host-side tests of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU (so all of this runs without one).

Pointers passed here are fake, 16-byte aligned, non-overlapping addresses: every call below must
return from validation with a negative status (or succeed with nothing to do) and never launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mamba_hip.h")


@pytest.fixture(scope="module")
def b():
    lib_path = os.path.join(ROOT, "paper_2506_01206_amd", "libmamba_hip.so")
    if not os.path.exists(lib_path):
        from paper_2506_01206_amd import build
        build.build()
    from paper_2506_01206_amd import binding
    return binding


def P(i):
    """i-th fake buffer: 1 TiB apart, 16-byte aligned, never dereferenced."""
    return (i + 1) << 40


def test_library_exports_every_declared_symbol(b):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(mamba2?_[a-z0-9_]+)\s*\(", text))
    assert declared == set(b.EXPORTS), declared ^ set(b.EXPORTS)
    raw = ctypes.CDLL(b.LIB_PATH)
    for name in declared:
        assert getattr(raw, name) is not None
    # the Python binding carries the same names
    for name in declared:
        assert callable(getattr(b, name))
    # second header: host-side tree search
    from paper_2506_01206_amd import tree_search
    text = open(os.path.join(ROOT, "include", "sd_tree_search.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(sd_[a-z0-9_]+)\s*\(", text))
    assert declared == set(tree_search.EXPORTS), declared ^ set(tree_search.EXPORTS)
    for name in declared:
        assert getattr(raw, name) is not None and callable(getattr(tree_search, name))


def test_binding_without_the_library_refuses_to_import(tmp_path, monkeypatch):
    """No fallback: a copy of the binding that finds no built library beside it raises on import."""
    monkeypatch.delenv("MAMBA_HIP_LIB", raising=False)
    import importlib.util
    import shutil
    shutil.copy(os.path.join(ROOT, "paper_2506_01206_amd", "binding.py"), tmp_path / "binding.py")
    spec = importlib.util.spec_from_file_location("binding_without_library", tmp_path / "binding.py")
    with pytest.raises(ImportError, match="libmamba_hip.so is missing"):
        spec.loader.exec_module(importlib.util.module_from_spec(spec))


def test_status_strings(b):
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6):
        s = b.mamba_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert b.mamba_status_string(-99) == "unknown status"
    assert b.mamba_status_string(1)            # a hipError_t text


def scan(b, x=P(0), dt=P(1), A=P(2), Bm=P(3), Cm=P(4), Dskip=P(5), z=P(6), bias=P(7), h0=P(8),
         out=P(9), hf=P(10), ws=P(11), ws_bytes=1 << 39, batch=1, L=4096, D=256, N=16, chunk=0,
         sp=1, io=1):
    return b.lib.mamba_scan_fwd(x, dt, A, Bm, Cm, Dskip, z, bias, h0, out, hf, ws, ws_bytes,
                                batch, L, D, N, chunk, sp, io, None)


def test_scan_validation(b):
    S = b.STATUS
    assert scan(b, x=None) == S["NULL_POINTER"]
    assert scan(b, A=None) == S["NULL_POINTER"]
    assert scan(b, out=None) == S["NULL_POINTER"]
    assert scan(b, L=-1) == S["BAD_SHAPE"]
    assert scan(b, batch=-2) == S["BAD_SHAPE"]
    assert scan(b, L=1 << 40, D=1 << 30) == S["BAD_SHAPE"]          # size overflow
    assert scan(b, N=17) == S["UNSUPPORTED"]
    assert scan(b, N=64) == S["UNSUPPORTED"]
    assert scan(b, io=7) == S["UNSUPPORTED"]
    assert scan(b, batch=70000, L=8, D=8) == S["UNSUPPORTED"]
    assert scan(b, x=P(0) + 8) == S["MISALIGNED"]
    assert scan(b, hf=P(10) + 4) == S["MISALIGNED"]
    assert scan(b, out=P(0)) == S["ALIAS"]                          # out == x
    assert scan(b, out=P(1) + 64) == S["ALIAS"]                     # out inside dt
    assert scan(b, hf=P(8) + 16) == S["ALIAS"]                      # h_final partly over h0
    assert scan(b, ws=None) == S["WORKSPACE"]                       # this shape is chunked
    assert scan(b, ws_bytes=16) == S["WORKSPACE"]
    assert scan(b, chunk=-1) == S["BAD_SHAPE"]
    # nothing to do: success without a launch
    assert scan(b, batch=0) == 0
    assert scan(b, D=0) == 0
    # a single chunk needs no workspace, so a missing one is not an error there; with an invalid
    # dtype the call still stops in validation
    assert b.mamba_scan_workspace_bytes(1, 4096, 256, 16, 4096) == 0
    assert b.mamba_scan_workspace_bytes(1, 4096, 256, 16, 1 << 40) == 0


def test_static_scan_validation(b):
    """The allocation-free scan validates like mamba_scan_fwd and refuses, before any HIP call, a shape whose chunk
    states do not fit the library's own buffer."""
    S = b.STATUS

    def sscan(x=P(0), dt=P(1), A=P(2), Bm=P(3), Cm=P(4), Dk=P(5), z=P(6), bias=P(7), h0=P(8), out=P(9), hf=P(10),
              batch=4, L=8192, D=4096, N=16, chunk=64, sp=1, io=1):
        return b.lib.mamba_scan_fwd_static(x, dt, A, Bm, Cm, Dk, z, bias, h0, out, hf, batch, L, D, N, chunk, sp, io, None)
    assert b.mamba_scan_workspace_bytes(4, 8192, 4096, 16, 64) > b.MAMBA_SCAN_STATIC_BYTES
    assert sscan() == S["WORKSPACE"]
    assert sscan(x=None) == S["NULL_POINTER"] and sscan(out=None) == S["NULL_POINTER"]
    assert sscan(L=-1) == S["BAD_SHAPE"] and sscan(N=17) == S["UNSUPPORTED"] and sscan(io=9) == S["UNSUPPORTED"]
    assert sscan(x=P(0) + 8) == S["MISALIGNED"] and sscan(out=P(0)) == S["ALIAS"]
    assert sscan(batch=0) == 0 and sscan(D=0) == 0
    header = open(HEADER).read()
    assert "#define MAMBA_SCAN_STATIC_BYTES (32u << 20)" in header and b.MAMBA_SCAN_STATIC_BYTES == 32 << 20


def test_strided_entry_points_validation(b):
    """Stride triples are host arrays of element counts {batch, token, channel}.  Everything is refused or found
    empty before any HIP call: negative strides, output layouts in which two elements coincide, byte ranges of an
    output and an input that overlap, base pointers not aligned to the element; NULL triples and triples that
    describe the contiguous layout fall through to the contiguous entry points' own rules."""
    S = b.STATUS
    I3 = ctypes.c_int64 * 3
    B, L, D, N = 2, 40, 24, 16

    def conv(x=P(0), xs=None, w=P(1), bias=P(2), cin=P(3), y=P(4), ys=None, cout=P(5), batch=B, L=L, D=D, K=4, io=1):
        return b.lib.mamba_conv1d_fwd_strided(x, xs, w, bias, cin, y, ys, cout, batch, L, D, K, 1, io, None)

    def scan(x=P(0), xs=None, dt=P(1), ds=None, A=P(2), Bm=P(3), Cm=P(4), Dk=P(5), z=P(6), zs=None, bias=P(7), h0=P(8),
             out=P(9), os_=None, hf=P(10), batch=B, L=L, D=D, N=N, io=1):
        return b.lib.mamba_scan_fwd_strided(x, xs, dt, ds, A, Bm, Cm, Dk, z, zs, bias, h0, out, os_, hf, None, 0,
                                            batch, L, D, N, 1, io, None)
    cm = I3(D * L, 1, L)                 # channel-major (batch, D, L)
    wide = I3(L * 2 * D, 2 * D, 1)       # a column range of rows twice as wide
    # what the contiguous calls refuse is refused here too, whatever the strides
    assert conv(io=7) == S["UNSUPPORTED"] and conv(K=9) == S["UNSUPPORTED"] and conv(L=-1) == S["BAD_SHAPE"]
    assert scan(io=7) == S["UNSUPPORTED"] and scan(N=-1) == S["BAD_SHAPE"] and scan(xs=cm, N=17) == S["UNSUPPORTED"]
    assert conv(batch=0, xs=cm) == 0 and scan(D=0, xs=cm) == 0
    # contiguous triples and 16-byte aligned bases: the contiguous entry point and its rules
    dense = I3(L * D, D, 1)
    assert conv(xs=dense, ys=dense, w=P(1) + 4) == S["MISALIGNED"]
    assert scan(xs=dense, ds=dense, zs=dense, os_=dense, out=P(0)) == S["ALIAS"]
    long = I3(32768 * 1536, 1536, 1)     # a shape the library cuts into time chunks: needs the workspace
    assert scan(xs=long, ds=long, zs=long, os_=long, L=32768, D=1536, batch=1) == S["WORKSPACE"]
    # strided path
    assert conv(xs=I3(D * L, -1, L)) == S["BAD_SHAPE"] and scan(ds=I3(-5, D, 1)) == S["BAD_SHAPE"]
    assert conv(xs=I3(1 << 62, 1 << 61, 1)) == S["BAD_SHAPE"]                      # extent overflows
    assert conv(ys=I3(D * L, 1, 1)) == S["BAD_SHAPE"] and scan(os_=I3(0, D, 1)) == S["BAD_SHAPE"]   # elements coincide
    assert scan(os_=I3(L * D, D - 1, 1)) == S["BAD_SHAPE"]
    assert conv(xs=cm, x=None) == S["NULL_POINTER"] and scan(os_=cm, A=None) == S["NULL_POINTER"]
    assert conv(xs=cm, x=P(0) + 1) == S["MISALIGNED"] and conv(xs=cm, w=P(1) + 4) == S["MISALIGNED"]
    assert scan(xs=cm, x=P(0) + 2, io=0) == S["MISALIGNED"] and scan(xs=cm, Bm=P(3) + 2) == S["MISALIGNED"]
    # ranges: an output inside the byte range an input spans is refused, also when no element coincides
    assert scan(xs=wide, os_=wide, out=P(0) + 2 * D) == S["ALIAS"]
    assert conv(xs=cm, y=P(0) + 2 * (L + 1)) == S["ALIAS"] and conv(xs=cm, cout=P(3)) == S["ALIAS"]
    assert conv(xs=cm, L=65535 * 128 + 1) == S["UNSUPPORTED"] and scan(xs=cm, batch=65536) == S["UNSUPPORTED"]


def test_scan_kernel_choice_by_shape(b):
    """The library's own choice of scan kernels is a pure function of the shape; an explicit chunk length always
    means time chunks (or one chunk)."""
    k = b.mamba_scan_kernel
    assert k(1, 32768, 1536, 16) == "chunked" and k(1, 2048, 1536, 16) == "lanes" and k(8, 8192, 4096, 16) == "direct"
    assert k(1, 256, 256, 16) == "lanes" and k(1, 2048, 1536, 8) == "chunked"      # lanes: 16 states only
    assert k(1, 2048, 1537, 16) == "chunked" and k(1, 32, 1536, 16) in ("single", "chunked")
    assert k(4, 8192, 4096, 16) == "direct" and k(4, 8192, 4100, 16) == "chunked"  # direct: 16-byte rows
    assert k(1, 2048, 1536, 16, 64) == "chunked" and k(1, 2048, 1536, 16, 2048) == "single"
    assert k(0, 10, 10, 16) == "" and k(1, 10, 10, 17) == "" and k(1, 10, 10, 16, -1) == ""
    for shape in ((1, 32768, 1536, 16), (1, 2048, 1536, 16), (8, 8192, 4096, 16), (1, 2048, 1536, 16, 64)):
        assert (b.mamba_scan_workspace_bytes(*shape) > 0) == (k(*shape) == "chunked")


def test_scan_workspace_query(b):
    w = b.mamba_scan_workspace_bytes
    assert w(0, 10, 10, 16, 0) == 0 and w(1, 0, 10, 16, 0) == 0 and w(1, 10, 10, 16, -1) == 0
    # explicit chunking: n_chunks slots of D*(N+1) floats per batch row
    assert w(2, 1000, 100, 16, 100) == 2 * 10 * 100 * 17 * 4
    assert w(2, 1001, 100, 16, 100) == 2 * 11 * 100 * 17 * 4
    assert w(1, 1000, 100, 16, 1000) == 0 and w(1, 1000, 100, 16, 5000) == 0
    # automatic chunking is a pure function of the shape, and grows no faster than L
    a = w(1, 32768, 1536, 16, 0)
    assert a == w(1, 32768, 1536, 16, 0) and a > 0
    assert a % (1536 * 17 * 4) == 0
    n_chunks = a // (1536 * 17 * 4)
    assert 2 <= n_chunks <= 32768 // 32
    # a batch-rich shape fills the chip without cutting time
    assert w(128, 4096, 4096, 16, 0) == 0
    # a very long batch-1 sequence: the library's own chunking stays within the 65535 chunks a launch can index
    # (an explicit chunk length that needs more is refused by the call itself)
    L = 256 * 65535 + 12345
    n = w(1, L, 8, 16, 0) // (8 * 17 * 4)
    assert 2 <= n <= 65535
    assert scan(b, L=L, D=8, batch=1, chunk=256, ws_bytes=1 << 40) == b.STATUS["UNSUPPORTED"]


def conv(b, x=P(0), w=P(1), bias=P(2), si=P(3), y=P(4), so=P(5), batch=2, L=100, D=64, K=4,
         silu=1, io=1):
    return b.lib.mamba_conv1d_fwd(x, w, bias, si, y, so, batch, L, D, K, silu, io, None)


def test_conv_validation(b):
    S = b.STATUS
    assert conv(b, x=None) == S["NULL_POINTER"]
    assert conv(b, w=None) == S["NULL_POINTER"]
    assert conv(b, y=None) == S["NULL_POINTER"]
    assert conv(b, K=1) == S["UNSUPPORTED"]
    assert conv(b, K=5) == S["UNSUPPORTED"]
    assert conv(b, io=2) == S["UNSUPPORTED"]
    assert conv(b, L=-1) == S["BAD_SHAPE"]
    assert conv(b, D=-1) == S["BAD_SHAPE"]
    assert conv(b, y=P(0)) == S["ALIAS"]
    assert conv(b, so=P(3) + 16) == S["ALIAS"]                      # partial state overlap
    assert conv(b, si=P(3) + 2, so=P(5)) == S["MISALIGNED"]
    assert conv(b, batch=0) == 0
    assert conv(b, L=0, so=None) == 0
    assert conv(b, L=0, si=P(3), so=P(3)) == 0                      # in place, nothing to shift


def step(b, ho=P(0), hi=P(1), par=P(2), x=P(3), dt=P(4), A=P(5), Bm=P(6), Cm=P(7), Dk=P(8), z=P(9),
         bias=P(10), out=P(11), n_out=8, n_in=4, D=64, N=16, sp=1, io=1):
    return b.lib.mamba_state_step(ho, hi, par, x, dt, A, Bm, Cm, Dk, z, bias, out, n_out, n_in, D, N,
                                  sp, io, None)


def test_step_validation(b):
    S = b.STATUS
    assert step(b, hi=None) == S["NULL_POINTER"]
    assert step(b, Cm=None) == S["NULL_POINTER"]
    assert step(b, par=None) == S["BAD_SHAPE"]                       # identity needs n_in == n_out
    assert step(b, n_in=0) == S["BAD_SHAPE"]
    assert step(b, n_out=-1) == S["BAD_SHAPE"]
    assert step(b, N=12) == S["UNSUPPORTED"]
    assert step(b, io=3) == S["UNSUPPORTED"]
    assert step(b, n_out=1 << 20) == S["UNSUPPORTED"]
    assert step(b, ho=P(1)) == S["ALIAS"]                            # in place only without parent
    assert step(b, ho=P(1) + 64, par=None, n_in=8) == S["ALIAS"]     # partial overlap never
    assert step(b, out=P(3)) == S["ALIAS"]
    assert step(b, x=P(3) + 2) == S["MISALIGNED"]
    assert step(b, n_out=0, n_in=4) == 0
    assert step(b, D=0) == 0


def conv_step(b, ho=P(0), hi=P(1), co=P(2), ci=P(3), par=P(4), x=P(5), cw=P(6), cb=P(7), dt=P(8), A=P(9), Bm=P(10),
              Cm=P(11), Dk=P(12), z=P(13), bias=P(14), out=P(15), xc=P(16), n_out=8, n_in=4, D=64, N=16, K=4, silu=1,
              sp=1, io=1):
    return b.lib.mamba_conv_state_step(ho, hi, co, ci, par, x, cw, cb, dt, A, Bm, Cm, Dk, z, bias, out, xc, n_out, n_in,
                                       D, N, K, silu, sp, io, None)


def test_conv_state_step_validation(b):
    S = b.STATUS
    assert conv_step(b, ci=None) == S["NULL_POINTER"]
    assert conv_step(b, cw=None) == S["NULL_POINTER"]
    assert conv_step(b, co=None) == S["NULL_POINTER"]
    assert conv_step(b, K=1) == S["UNSUPPORTED"]
    assert conv_step(b, K=5) == S["UNSUPPORTED"]
    assert conv_step(b, N=12) == S["UNSUPPORTED"]
    assert conv_step(b, io=7) == S["UNSUPPORTED"]
    assert conv_step(b, par=None) == S["BAD_SHAPE"]                  # identity needs n_in == n_out
    assert conv_step(b, n_in=0) == S["BAD_SHAPE"]
    assert conv_step(b, ho=P(1)) == S["ALIAS"]                       # in place only without a parent index
    assert conv_step(b, co=P(3)) == S["ALIAS"]
    assert conv_step(b, co=P(3) + 32, par=None, n_in=8) == S["ALIAS"]   # partial overlap never
    assert conv_step(b, xc=P(15)) == S["ALIAS"]                      # two outputs on each other
    assert conv_step(b, out=P(5)) == S["ALIAS"]                      # output on an input
    assert conv_step(b, co=P(1)) == S["ALIAS"]                       # new windows on the old SSM state
    assert conv_step(b, x=P(5) + 2) == S["MISALIGNED"]
    assert conv_step(b, xc=None, cb=None, Dk=None, z=None, bias=None, n_out=0) == 0
    assert conv_step(b, D=0) == 0


def fork(b, cd=P(0), cs=P(1), sd=P(2), ss=P(3), par=P(4), nl=24, n_out=8, n_in=4, D=64, N=16, K=4,
         io=1):
    return b.lib.mamba_state_fork(cd, cs, sd, ss, par, nl, n_out, n_in, D, N, K, io, None)


def test_fork_validation(b):
    S = b.STATUS
    assert fork(b, par=None) == S["NULL_POINTER"]
    assert fork(b, cd=None) == S["NULL_POINTER"]                     # half of the conv pair
    assert fork(b, ss=None) == S["NULL_POINTER"]                     # half of the ssm pair
    assert fork(b, n_in=0) == S["BAD_SHAPE"]
    assert fork(b, nl=-1) == S["BAD_SHAPE"]
    assert fork(b, io=5) == S["UNSUPPORTED"]
    assert fork(b, n_out=1 << 17) == S["UNSUPPORTED"]
    assert fork(b, cd=P(1)) == S["ALIAS"]
    assert fork(b, sd=P(3) + 1024) == S["ALIAS"]
    assert fork(b, cs=P(1) + 4) == S["MISALIGNED"]
    assert fork(b, n_out=0) == 0
    assert fork(b, nl=0) == 0
    assert fork(b, cd=None, cs=None, sd=None, ss=None) == 0


def read_golden_trees():
    rows = []
    with open(os.path.join(ROOT, "tests", "golden", "tree_configs.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                t, bsz = line.split("|")
                rows.append((tuple(int(v) for v in t.split(",")), [int(v) for v in bsz.split(",")]))
    return rows


def test_tree_plan_matches_the_paper_trees(b):
    """Batch sizes B_i = N_1..N_i of the trees the paper prints, one cache per distinct batch size
    (Sec. 4.1), all inside one slab without overlap."""
    import torch
    nl, D, N, K = 24, 1536, 16, 4
    for tree, sizes in read_golden_trees():
        p = b.mamba_tree_plan(tree, nl, D, N, K, torch.bfloat16)
        assert p.gamma == len(tree)
        assert [p.batch[i] for i in range(len(tree) + 1)] == [1] + sizes
        distinct = sorted(set([1] + sizes))
        assert p.n_caches == len(distinct)
        assert [p.cache_batch[c] for c in range(p.n_caches)] == distinct
        spans = []
        for c in range(p.n_caches):
            bs = p.cache_batch[c]
            spans.append((p.conv_offset[c], nl * bs * D * (K - 1) * 2))
            spans.append((p.ssm_offset[c], nl * bs * D * N * 4))
        for i, n_i in enumerate(tree, start=1):
            assert p.cache_batch[p.cache_of_depth[i]] == sizes[i - 1]
            if n_i == 1:
                assert p.parent_offset[i] == -1 and p.cache_of_depth[i] == p.cache_of_depth[i - 1]
            else:
                assert p.cache_of_depth[i] == p.cache_of_depth[i - 1] + 1
                spans.append((p.parent_offset[i], sizes[i - 1] * 4))
        spans.sort()
        for (o, n), (o2, _) in zip(spans, spans[1:]):
            assert o % 256 == 0 and o + n <= o2
        assert spans[-1][0] + spans[-1][1] <= p.total_bytes
        assert p.total_bytes - sum(n for _, n in spans) < 256 * len(spans)     # only alignment padding


def test_tree_plan_validation(b):
    import ctypes
    S = b.STATUS
    plan = b.TreePlan()

    def call(tree, gamma=None, nl=2, D=64, N=16, K=4, io=1, out=plan):
        arr = (ctypes.c_int32 * max(len(tree), 1))(*tree)
        return b.lib.mamba_tree_plan(arr, len(tree) if gamma is None else gamma, nl, D, N, K, io,
                                     ctypes.byref(out) if out is not None else None)
    assert call([3, 2, 1]) == 0
    assert call([]) == S["BAD_SHAPE"]
    assert call([2] * 17) == S["BAD_SHAPE"]                   # deeper than MAMBA_MAX_DEPTH
    assert call([3, 0, 2]) == S["BAD_SHAPE"]
    assert call([3, -1]) == S["BAD_SHAPE"]
    assert call([256, 256, 2]) == S["UNSUPPORTED"]            # 131072 branches
    assert call([2], N=5) == S["UNSUPPORTED"]
    assert call([2], K=7) == S["UNSUPPORTED"]
    assert call([2], io=9) == S["UNSUPPORTED"]
    assert call([2], nl=-1) == S["BAD_SHAPE"]
    assert call([2], nl=1 << 40, D=1 << 30) == S["BAD_SHAPE"]
    assert b.lib.mamba_tree_plan(None, 1, 1, 8, 16, 4, 1, ctypes.byref(plan)) == S["NULL_POINTER"]
    # parents: a plan made for another tree is refused before anything is launched
    assert call([3, 2, 1]) == 0
    other = (ctypes.c_int32 * 3)(3, 1, 2)
    assert b.lib.mamba_tree_parents(P(0), ctypes.byref(plan), other, None) == S["BAD_SHAPE"]
    assert b.lib.mamba_tree_parents(None, ctypes.byref(plan), other, None) == S["NULL_POINTER"]
    assert b.lib.mamba_tree_parents(P(0) + 4, ctypes.byref(plan), other, None) == S["MISALIGNED"]


def ssd(b, x=P(0), dt=P(1), A=P(2), Bm=P(3), Cm=P(4), Dskip=P(5), z=P(6), bias=P(7), h0=P(8), out=P(9), hf=P(10),
        ws=P(11), ws_bytes=1 << 39, batch=1, L=4096, H=24, Pd=64, N=128, sp=1, io=1):
    return b.lib.mamba2_ssd_fwd(x, dt, A, Bm, Cm, Dskip, z, bias, h0, out, hf, ws, ws_bytes, batch, L, H, Pd, N, sp, io, None)


def test_ssd_validation(b):
    """Every rejection of the scalar-decay scan and step happens on the host, before any launch."""
    S = b.STATUS
    assert ssd(b, x=None) == S["NULL_POINTER"] and ssd(b, Cm=None) == S["NULL_POINTER"] and ssd(b, out=None) == S["NULL_POINTER"]
    assert ssd(b, L=-1) == S["BAD_SHAPE"] and ssd(b, H=-3) == S["BAD_SHAPE"]
    assert ssd(b, L=1 << 40, H=1 << 30) == S["BAD_SHAPE"]                      # size overflow
    assert ssd(b, Pd=32) == S["UNSUPPORTED"] and ssd(b, N=16) == S["UNSUPPORTED"] and ssd(b, N=256) == S["UNSUPPORTED"]
    assert ssd(b, io=0) == S["UNSUPPORTED"]                                    # float32 I/O: the products run in bf16
    assert ssd(b, batch=70000, L=8, H=1) == S["UNSUPPORTED"]
    assert ssd(b, x=P(0) + 2) == S["MISALIGNED"] and ssd(b, ws=P(11) + 8) == S["MISALIGNED"]
    assert ssd(b, ws=None) == S["WORKSPACE"] and ssd(b, ws_bytes=1000) == S["WORKSPACE"]
    assert ssd(b, out=P(0)) == S["ALIAS"] and ssd(b, out=P(6)) == S["ALIAS"] and ssd(b, ws=P(9)) == S["ALIAS"]
    assert ssd(b, batch=0) == 0 and ssd(b, H=0) == 0
    need = b.lib.mamba2_ssd_workspace_bytes(1, 4096, 24, 64, 128)
    assert need > 0 and ssd(b, ws_bytes=need - 1) == S["WORKSPACE"]
    assert b.lib.mamba2_ssd_workspace_bytes(1, 4096, 24, 32, 128) == 0 and b.lib.mamba2_ssd_workspace_bytes(0, 64, 1, 64, 64) == 0
    # the workspace holds one state per segment, not per chunk: it stays small for long sequences
    assert b.lib.mamba2_ssd_workspace_bytes(1, 1 << 20, 24, 64, 128) < 64 << 20

    def step(h_out=P(0), h_in=P(1), par=P(2), x=P(3), dt=P(4), A=P(5), Bm=P(6), Cm=P(7), Dskip=P(8), z=P(9), bias=P(10),
             out=P(11), n_out=8, n_in=4, H=24, Pd=64, N=128, sp=1, io=1):
        return b.lib.mamba2_state_step(h_out, h_in, par, x, dt, A, Bm, Cm, Dskip, z, bias, out, n_out, n_in, H, Pd, N, sp, io, None)
    assert step(h_in=None) == S["NULL_POINTER"] and step(out=None) == S["NULL_POINTER"]
    assert step(n_out=-1) == S["BAD_SHAPE"] and step(par=None) == S["BAD_SHAPE"]              # no parents: n_in must equal n_out
    assert step(n_in=0) == S["BAD_SHAPE"]
    assert step(N=32) == S["UNSUPPORTED"] and step(Pd=128) == S["UNSUPPORTED"] and step(io=5) == S["UNSUPPORTED"]
    assert step(n_out=70000) == S["UNSUPPORTED"]
    assert step(par=P(2) + 4) == S["MISALIGNED"]
    assert step(h_out=P(1)) == S["ALIAS"]                                                     # in place only without parents
    assert step(out=P(3)) == S["ALIAS"]
    assert step(n_out=0) == 0


def _block_params(b, dm=768, D=1536, N=16, R=48, K=4, **ptrs):
    names = ["norm_w", "in_proj_w", "conv_w", "conv_b", "x_proj_w", "dt_proj_w", "dt_bias", "A", "Dskip", "out_proj_w"]
    vals = {n: P(20 + i) for i, n in enumerate(names)}
    vals.update(ptrs)
    return b.BlockParams(dm, D, N, R, K, 1e-5, *[vals[n] for n in names])


def test_block_validation_and_workspace(b):
    """The whole-block entry points check parameters, pointers, aliasing and the workspace on the host."""
    S = b.STATUS
    ws_bytes = b.lib.mamba_block_workspace_bytes
    p = _block_params(b)
    need_prefill = ws_bytes(ctypes.byref(p), 1, 2048)
    need_step = ws_bytes(ctypes.byref(p), 12, 1)
    assert need_prefill >= 4 * 2048 * 1536 * 2 and need_step >= 4 * 12 * 1536 * 2
    # one token on a few rows also holds the partial sums of the x projection: (d_inner / 32, rows, dt_rank + 2 N) floats
    assert need_step >= 4 * 12 * 1536 * 2 + (1536 // 32) * 12 * 80 * 4
    assert ws_bytes(ctypes.byref(p), 12, 1) < ws_bytes(ctypes.byref(p), 24, 1)
    assert ws_bytes(ctypes.byref(p), 0, 1) == 0 and ws_bytes(ctypes.byref(p), 1, 0) == 0
    assert ws_bytes(ctypes.byref(_block_params(b, N=5)), 1, 64) == 0 and ws_bytes(ctypes.byref(_block_params(b, dm=772)), 1, 64) == 0

    # where the stage tensors lie: seven disjoint bf16 tensors inside the workspace, 256-byte aligned, dt first
    off = (ctypes.c_int64 * 7)()
    layout = b.lib.mamba_block_workspace_layout
    assert layout(ctypes.byref(p), 1, 2048, off) == 0
    sizes = [2048 * 1536 * 2] * 4 + [2048 * 48 * 2, 2048 * 16 * 2, 2048 * 16 * 2]
    spans = sorted((int(o), int(o) + n) for o, n in zip(off, sizes))
    assert off[0] == 0 and all(o % 256 == 0 for o in off) and spans[-1][1] <= need_prefill
    assert all(a[1] <= c[0] for a, c in zip(spans, spans[1:]))
    assert layout(ctypes.byref(p), 1, 2048, None) == S["NULL_POINTER"] and layout(ctypes.byref(p), 0, 5, off) == S["BAD_SHAPE"]
    assert layout(ctypes.byref(_block_params(b, N=5)), 1, 64, off) == S["UNSUPPORTED"]

    def fwd(p=p, hid=P(0), out=P(1), ci=P(2), co=P(3), h0=P(4), hf=P(5), ws=P(6), wsb=need_prefill, batch=1, L=2048):
        return b.lib.mamba_block_fwd(ctypes.byref(p), hid, out, ci, co, h0, hf, ws, wsb, batch, L, None)
    assert fwd(hid=None) == S["NULL_POINTER"] and fwd(out=None) == S["NULL_POINTER"]
    assert fwd(p=_block_params(b, in_proj_w=None)) == S["NULL_POINTER"]
    assert fwd(batch=-1) == S["BAD_SHAPE"] and fwd(p=_block_params(b, R=0)) == S["BAD_SHAPE"]
    assert fwd(p=_block_params(b, N=5)) == S["UNSUPPORTED"] and fwd(p=_block_params(b, K=9)) == S["UNSUPPORTED"]
    assert fwd(p=_block_params(b, dm=8192)) == S["UNSUPPORTED"]
    assert fwd(hid=P(0) + 2) == S["MISALIGNED"] and fwd(p=_block_params(b, A=P(27) + 4)) == S["MISALIGNED"]
    assert fwd(ws=None) == S["WORKSPACE"] and fwd(wsb=need_prefill - 1) == S["WORKSPACE"]
    assert fwd(batch=0) == 0 and fwd(L=0) == 0

    def step(p=p, hid=P(0), out=P(1), cs=P(2), cd=P(3), ss=P(4), sd=P(5), par=P(7), ws=P(6), wsb=need_step, n_out=12, n_in=6):
        return b.lib.mamba_block_step(ctypes.byref(p), hid, out, cs, cd, ss, sd, par, ws, wsb, n_out, n_in, None)
    assert step(hid=None) == S["NULL_POINTER"] and step(sd=None) == S["NULL_POINTER"]
    assert step(n_out=-1) == S["BAD_SHAPE"] and step(n_in=0) == S["BAD_SHAPE"]
    assert step(par=None) == S["BAD_SHAPE"]                                     # no parents: in place, same batch
    assert step(cd=P(2)) == S["ALIAS"] and step(sd=P(4)) == S["ALIAS"]          # children never overwrite their parents
    assert step(par=P(7) + 4) == S["MISALIGNED"] and step(ws=P(6) + 8) == S["MISALIGNED"]
    assert step(ws=None) == S["WORKSPACE"] and step(wsb=need_step - 1) == S["WORKSPACE"]
    assert step(out=P(2)) == S["ALIAS"] and step(ws=P(4)) == S["ALIAS"]
    assert step(n_out=0) == 0 and step(n_out=70000, n_in=70000, wsb=1 << 40) == S["UNSUPPORTED"]


def test_linear_norm_and_vocabulary_validation(b):
    S = b.STATUS

    def lin(x=P(0), w=P(1), bias=P(2), res=None, o0=P(3), w0=3072, o1=None, w1=0, o2=None, w2=0, M=64, K=768, io=1):
        return b.lib.mamba_linear_fwd(x, w, bias, res, o0, w0, o1, w1, o2, w2, M, K, io, None)
    assert lin(x=None) == S["NULL_POINTER"] and lin(o0=None) == S["NULL_POINTER"]
    assert lin(M=-1) == S["BAD_SHAPE"] and lin(w0=-8) == S["BAD_SHAPE"]
    assert lin(io=0) == S["UNSUPPORTED"] and lin(K=770) == S["UNSUPPORTED"]
    assert lin(x=P(0) + 2) == S["MISALIGNED"]
    assert lin(o0=P(0)) == S["ALIAS"] and lin(o0=P(1)) == S["ALIAS"]
    assert lin(M=0) == 0

    def norm(x=P(0), w=P(1), y=P(2), M=16, C=768, eps=1e-5, io=1):
        return b.lib.mamba_rmsnorm_fwd(x, w, y, M, C, eps, io, None)
    assert norm(x=None) == S["NULL_POINTER"] and norm(M=-2) == S["BAD_SHAPE"] and norm(eps=-1.0) == S["BAD_SHAPE"]
    assert norm(C=772) == S["UNSUPPORTED"] and norm(C=8192) == S["UNSUPPORTED"] and norm(io=0) == S["UNSUPPORTED"]
    assert norm(y=P(2) + 4) == S["MISALIGNED"] and norm(y=P(0) + 16) == S["ALIAS"] and norm(M=0) == 0

    def emb(tok=P(0), table=P(1), out=P(2), M=12, V=50280, dm=768, io=1):
        return b.lib.mamba_embedding_fwd(tok, table, out, M, V, dm, io, None)
    assert emb(tok=None) == S["NULL_POINTER"] and emb(V=0) == S["BAD_SHAPE"] and emb(dm=772) == S["UNSUPPORTED"]
    assert emb(io=0) == S["UNSUPPORTED"] and emb(out=P(1)) == S["ALIAS"] and emb(M=0) == 0

    def topk(logits=P(0), idx=P(1), val=P(2), M=12, V=50280, k=3, io=1):
        return b.lib.mamba_topk_fwd(logits, idx, val, M, V, k, io, None)
    assert topk(idx=None) == S["NULL_POINTER"] and topk(M=-1) == S["BAD_SHAPE"]
    assert topk(k=0) == S["UNSUPPORTED"] and topk(k=9) == S["UNSUPPORTED"] and topk(V=(1 << 25) + 1) == S["UNSUPPORTED"]
    assert topk(io=0) == S["UNSUPPORTED"] and topk(val=P(2) + 4) == S["MISALIGNED"] and topk(idx=P(0)) == S["ALIAS"]
    assert topk(M=0) == 0
