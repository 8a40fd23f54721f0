"""GPU parity: every entry point of the C ABI against the fp64 oracle, element by element, on the
same seeded inputs; plus the invariants that hold at any size (scan == repeated steps, chunked
== unchunked, fused fork+step == fork then step bit for bit, run-to-run determinism)."""
import sys

import numpy as np
import pytest
import torch

import oracle
from oracle import tree as oracle_tree
from paper_2506_01206_amd import synth
from gpu_util import DEV, TOL, W, assert_close, dev_case, oracle_scan, to_dev, to_host, values

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def m():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2506_01206_amd import binding
    return binding


@pytest.fixture(autouse=True)
def announce(request):
    print("\n[gpu-case] %s" % request.node.nodeid, flush=True)
    sys.stdout.flush()
    yield
    torch.cuda.synchronize()


def say(**kw):
    print("    " + " ".join("%s=%s" % kv for kv in kw.items()), flush=True)


# ------------------------------------------------------------------------------------ conv1d
def run_conv(m, c, state_in=None, apply_silu=True, want_state=True):
    d = dev_case(c, ("x", "conv_w", "conv_bias"))
    y, st = m.mamba_conv1d_fwd(d["x"], d["conv_w"], d["conv_bias"], to_dev(state_in),
                               apply_silu=apply_silu, want_state=want_state)
    return to_host(y), to_host(st)


def check_conv(m, c, state_in=None, apply_silu=True):
    y, st = run_conv(m, c, state_in, apply_silu)
    ry, rst = oracle.conv1d_fwd(W(c["x"]), W(c["conv_w"]), W(c["conv_bias"]), W(state_in), apply_silu)
    assert_close(values(y), ry, TOL[c["io"]], "conv y")
    # the carried state is a verbatim copy of inputs: exact in the storage dtype
    assert np.array_equal(values(st), rst), "conv state"


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("K", [2, 3, 4])
@pytest.mark.parametrize("B,L,D", [(1, 1, 8), (2, 3, 17), (1, 63, 64), (3, 65, 100), (1, 257, 256),
                                   (2, 1000, 24), (1, 2, 1)])
def test_conv_shapes(m, io, K, B, L, D):
    say(io=io, K=K, B=B, L=L, D=D)
    c = synth.prefill_case(B, L, D, 16, K, io, seed=1000 + L + D + K)
    rng = np.random.default_rng(7)
    c["conv_bias"] = rng.standard_normal(D).astype(np.float32)
    st0 = synth.to_io(rng.standard_normal((B, D, K - 1)).astype(np.float32), io)
    check_conv(m, c, None, True)
    check_conv(m, c, st0, False)


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
def test_conv_carry_and_in_place_state(m, io):
    B, L, D, K = 2, 150, 64, 4
    c = synth.prefill_case(B, L, D, 16, K, io, seed=77)
    d = dev_case(c, ("x", "conv_w", "conv_bias"))
    y_full, st_full = m.mamba_conv1d_fwd(d["x"], d["conv_w"], d["conv_bias"])
    # token by token with the window updated in place (the decode-time use)
    state = torch.zeros((B, D, K - 1), dtype=d["x"].dtype, device=DEV)
    ys = []
    for t in range(L):
        xt = d["x"][:, t:t + 1].contiguous()
        yt, _ = m.mamba_conv1d_fwd(xt, d["conv_w"], d["conv_bias"], conv_state_in=state,
                                   conv_state_out=state)
        ys.append(yt)
    y_steps = torch.cat(ys, dim=1)
    assert torch.equal(y_steps, y_full)          # same arithmetic, same order: bit-identical
    assert torch.equal(state, st_full)
    # two pieces with a carried state
    y1, s1 = m.mamba_conv1d_fwd(d["x"][:, :70].contiguous(), d["conv_w"], d["conv_bias"])
    y2, s2 = m.mamba_conv1d_fwd(d["x"][:, 70:].contiguous(), d["conv_w"], d["conv_bias"], conv_state_in=s1)
    assert torch.equal(torch.cat([y1, y2], 1), y_full) and torch.equal(s2, st_full)
    # L == 0 passes the state through
    e = d["x"][:, :0].contiguous()
    _, s0 = m.mamba_conv1d_fwd(e, d["conv_w"], d["conv_bias"], conv_state_in=s1)
    assert torch.equal(s0, s1)
    _, sz = m.mamba_conv1d_fwd(e, d["conv_w"], d["conv_bias"])
    assert torch.count_nonzero(sz.float()) == 0


# ------------------------------------------------------------------------------------ scan
def run_scan(m, c, h0=None, chunk_len=0, **kw):
    d = dev_case(c)
    args = dict(x=d["x"], dt=d["dt"], A=d["A"], Bm=d["Bm"], Cm=d["Cm"], Dskip=d["Dskip"], z=d["z"],
                dt_bias=d["dt_bias"], h0=to_dev(h0), chunk_len=chunk_len)
    args.update(kw)
    out, hf = m.mamba_scan_fwd(**args)
    return to_host(out), to_host(hf)


def check_scan(m, c, h0=None, chunk_len=0, what="scan", **kw):
    out, hf = run_scan(m, c, h0, chunk_len, **kw)
    okw = {}
    for k in ("Dskip", "z", "dt_bias"):
        if k in kw and kw[k] is None:
            okw[k] = None
    if "dt_softplus" in kw:
        okw["dt_softplus"] = kw["dt_softplus"]
    ro, rh = oracle_scan(c, h0=None if h0 is None else h0.astype(np.float64), **okw)
    e1 = assert_close(values(out), ro, TOL[c["io"]], what + " out")
    e2 = assert_close(hf, rh, TOL[c["io"]], what + " h_final")
    return e1, e2


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("L", [1, 2, 3, 63, 64, 65, 255, 257, 1000])
@pytest.mark.parametrize("D", [1, 17, 64, 100, 256])
def test_scan_shapes(m, io, L, D):
    say(io=io, L=L, D=D)
    B, N = (2 if L < 300 else 1), 16
    c = synth.prefill_case(B, L, D, N, 4, io, seed=L * 1000 + D)
    h0 = np.random.default_rng(L + D).standard_normal((B, D, N)).astype(np.float32)
    check_scan(m, c, h0=h0)
    if L in (65, 257, 1000):
        for cl in (1, 7, 64, 100):
            check_scan(m, c, h0=h0, chunk_len=cl, what="scan chunk_len=%d" % cl)


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("N", [4, 8, 16, 32])
def test_scan_state_sizes_and_random_A(m, io, N):
    say(io=io, N=N)
    c = synth.prefill_case(2, 300, 96, N, 4, io, seed=500 + N, random_A=True)
    check_scan(m, c)
    check_scan(m, c, chunk_len=64, what="chunked")
    c2 = synth.prefill_case(1, 300, 33, N, 4, io, seed=600 + N, random_A=True)   # odd D
    check_scan(m, c2, chunk_len=50, what="odd D chunked")


@pytest.mark.parametrize("N", [4, 8, 16, 32])
@pytest.mark.parametrize("L,chunk_len", [(640, 16), (1000, 5), (1200, 3)])
def test_scan_carry_variants(m, N, L, chunk_len):
    """The three carry kernels between the passes: 40 slots (four states per lane), 200 slots (two states per lane),
    400 slots (the looped variant), for every state size and an odd channel count."""
    say(N=N, L=L, chunk_len=chunk_len)
    c = synth.prefill_case(2, L, 66, N, 4, synth.F32, seed=3000 + N + L, random_A=True)
    h0 = np.random.default_rng(N + L).standard_normal((2, 66, N)).astype(np.float32)
    check_scan(m, c, h0=h0, chunk_len=chunk_len, what="carry over %d slots" % ((L + chunk_len - 1) // chunk_len))


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("N", [4, 8, 16, 32])
@pytest.mark.parametrize("B,L,D", [(56, 1, 256), (56, 31, 256), (28, 65, 512), (56, 100, 200), (224, 129, 64), (230, 7, 8)])
def test_scan_single_pass_shapes(m, io, N, B, L, D):
    """Shapes with enough independent channels that the library walks every token once (no time chunks, no
    workspace): tile tails, a channel block that is only partly there (D = 200, D = 8), every state size."""
    say(io=io, N=N, B=B, L=L, D=D)
    assert m.mamba_scan_workspace_bytes(B, L, D, N) == 0 and m.mamba_scan_kernel(B, L, D, N) == "direct"
    c = synth.prefill_case(B, L, D, N, 4, io, seed=40000 + N + L + D, random_A=True)
    h0 = np.random.default_rng(N + L + D).standard_normal((B, D, N)).astype(np.float32)
    check_scan(m, c, h0=h0, what="single pass")
    if L == 100:
        check_scan(m, c, what="single pass, zero state, no gate", z=None)
        check_scan(m, c, h0=h0, what="single pass, no skip, no bias", Dskip=None, dt_bias=None)
        c3 = dict(c)
        c3["dt"] = synth.to_io(np.abs(synth.io_values(c["dt"], io)) + 0.01, io)
        check_scan(m, c3, h0=h0, dt_softplus=False, dt_bias=None, what="single pass, delta given directly")
        # the same inputs cut in time take the two-pass kernels: same result within the tolerance of each
        o1, h1 = run_scan(m, c, h0=h0)
        o2, h2 = run_scan(m, c, h0=h0, chunk_len=16)
        assert_close(values(o1), values(o2), 2 * TOL[io], "single pass vs chunked out")
        assert_close(h1, h2, 2 * TOL[io], "single pass vs chunked state")
        # in-place state
        d = dev_case(c)
        st = to_dev(h0).clone()
        m.mamba_scan_fwd(d["x"], d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"], h0=st, h_final=st)
        assert np.array_equal(to_host(st), h1)


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("B,L,D", [(1, 64, 576), (1, 513, 576), (2, 1000, 290), (1, 1030, 580), (3, 700, 198),
                                   (1, 1537, 1536), (16, 100, 36)])
def test_scan_time_across_lanes_shapes(m, io, B, L, D):
    """One or a few sequences of a narrow layer with 16 states: the library scans time across the lanes of a
    wavefront (super-steps of 512 tokens, no chunks, no workspace).  Ragged last super-step, several super-steps,
    channel counts that leave the last workgroup 2 or 4 channels of its own, a nonzero incoming state."""
    say(io=io, B=B, L=L, D=D)
    N = 16
    assert m.mamba_scan_workspace_bytes(B, L, D, N) == 0 and m.mamba_scan_kernel(B, L, D, N) == "lanes"
    c = synth.prefill_case(B, L, D, N, 4, io, seed=50000 + L + D, random_A=True)
    h0 = np.random.default_rng(L + D).standard_normal((B, D, N)).astype(np.float32)
    check_scan(m, c, h0=h0, what="lanes")
    if L in (513, 1000):
        check_scan(m, c, what="lanes, zero state, no gate", z=None)
        check_scan(m, c, h0=h0, what="lanes, no skip, no bias", Dskip=None, dt_bias=None)
        c3 = dict(c)
        c3["dt"] = synth.to_io(np.abs(synth.io_values(c["dt"], io)) + 0.01, io)
        check_scan(m, c3, h0=h0, dt_softplus=False, dt_bias=None, what="lanes, delta given directly")
        c4 = dict(c)
        c4["A"] = np.zeros_like(c["A"])
        check_scan(m, c4, h0=h0, what="lanes, A = 0")
        # the same inputs cut into time chunks take the two-pass kernels
        o1, h1 = run_scan(m, c, h0=h0)
        o2, h2 = run_scan(m, c, h0=h0, chunk_len=100)
        assert_close(values(o1), values(o2), 2 * TOL[io], "lanes vs chunked out")
        assert_close(h1, h2, 2 * TOL[io], "lanes vs chunked state")
        # in-place state, and run-to-run determinism
        d = dev_case(c)
        st = to_dev(h0).clone()
        o3, _ = m.mamba_scan_fwd(d["x"], d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"], h0=st, h_final=st)
        assert np.array_equal(to_host(st), h1) and np.array_equal(to_host(o3), o1)


def test_scan_time_across_lanes_delta_to_zero_keeps_state(m):
    # dt = -1e4 under softplus: every decay is exactly 1 and every input term 0, also through the scan over lanes
    c = synth.prefill_case(1, 700, 576, 16, 4, synth.F32, seed=19)
    c["dt"] = np.full_like(c["dt"], -1e4)
    h0 = np.random.default_rng(2).standard_normal((1, 576, 16)).astype(np.float32)
    _, hf = run_scan(m, c, h0=h0)
    assert np.array_equal(hf, h0)


# ------------------------------------------------------------------------------------ other layouts
def channel_major(t):
    """A (B,L,D) device tensor re-stored as (B,D,L) and handed back as its (B,L,D) view."""
    return t.transpose(1, 2).contiguous().transpose(1, 2)


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("B,L,D,N", [(2, 150, 100, 16), (1, 1, 7, 4), (3, 33, 64, 8), (1, 700, 130, 32)])
def test_scan_strided_layouts(m, io, B, L, D, N):
    """mamba_scan_fwd_strided: channel-major tensors, x and z as the two halves of one wide tensor, an output
    written into a wider buffer; each against the oracle on the logical (B,L,D) arrays.  Strides that describe the
    contiguous layout give the bits of mamba_scan_fwd."""
    say(io=io, B=B, L=L, D=D, N=N)
    c = synth.prefill_case(B, L, D, N, 4, io, seed=61000 + L + D, random_A=True)
    h0 = np.random.default_rng(L + D).standard_normal((B, D, N)).astype(np.float32)
    ro, rh = oracle_scan(c, h0=h0.astype(np.float64))
    d = dev_case(c)
    fixed = dict(A=d["A"], Bm=d["Bm"], Cm=d["Cm"], Dskip=d["Dskip"], dt_bias=d["dt_bias"], h0=to_dev(h0))
    # channel-major inputs and output
    out_cm = torch.empty((B, D, L), dtype=d["x"].dtype, device=DEV).transpose(1, 2)
    o, hf = m.mamba_scan_fwd_strided(channel_major(d["x"]), channel_major(d["dt"]), z=channel_major(d["z"]), out=out_cm, **fixed)
    assert o.stride() == (D * L, 1, L)
    assert_close(values(to_host(o.contiguous())), ro, TOL[io], "channel-major out")
    assert_close(to_host(hf), rh, TOL[io], "channel-major h_final")
    # x | z side by side in one (B, L, 2D) tensor, dt contiguous, out into columns D/2.. of a wider buffer
    xz = torch.cat([d["x"], d["z"]], dim=2)
    wide = torch.full((B, L, 2 * D + 3), 7.0, dtype=d["x"].dtype, device=DEV)
    o2, hf2 = m.mamba_scan_fwd_strided(xz[..., :D], d["dt"], z=xz[..., D:], out=wide[..., 3:3 + D], **fixed)
    assert_close(values(to_host(o2.contiguous())), ro, TOL[io], "packed x|z out")
    assert_close(to_host(hf2), rh, TOL[io], "packed x|z h_final")
    assert torch.all(wide[..., :3] == 7.0) and torch.all(wide[..., 3 + D:] == 7.0)      # nothing outside the view
    assert torch.equal(o2.contiguous(), o.contiguous()) and torch.equal(hf2, hf)         # one kernel, one order
    # no gate, no state in or out
    o3, none = m.mamba_scan_fwd_strided(channel_major(d["x"]), d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"],
                                        dt_bias=d["dt_bias"], want_state=False)
    ro3, _ = oracle_scan(c, z=None)
    assert none is None
    assert_close(values(to_host(o3)), ro3, TOL[io], "no gate out")
    # contiguous strides: the tuned kernels, bit for bit
    o4, hf4 = m.mamba_scan_fwd_strided(d["x"], d["dt"], z=d["z"], **fixed)
    o5, hf5 = m.mamba_scan_fwd(d["x"], d["dt"], z=d["z"], **fixed)
    assert torch.equal(o4, o5) and torch.equal(hf4, hf5)


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("K", [2, 4])
@pytest.mark.parametrize("B,L,D", [(2, 150, 100), (1, 2, 9), (3, 300, 64), (1, 1, 1)])
def test_conv_strided_layouts(m, io, K, B, L, D):
    """mamba_conv1d_fwd_strided on channel-major tensors and on a column range of a wider tensor, with a carried
    window; outputs within tolerance of the oracle and bit-identical to the contiguous call (same order of
    operations), carried states exact."""
    say(io=io, K=K, B=B, L=L, D=D)
    c = synth.prefill_case(B, L, D, 16, K, io, seed=62000 + L + D + K)
    rng = np.random.default_rng(9)
    c["conv_bias"] = rng.standard_normal(D).astype(np.float32)
    st0 = synth.to_io(rng.standard_normal((B, D, K - 1)).astype(np.float32), io)
    ry, rst = oracle.conv1d_fwd(W(c["x"]), W(c["conv_w"]), W(c["conv_bias"]), W(st0), True)
    d = dev_case(c, ("x", "conv_w", "conv_bias"))
    y_ref, st_ref = m.mamba_conv1d_fwd(d["x"], d["conv_w"], d["conv_bias"], to_dev(st0))
    y_cm = torch.empty((B, D, L), dtype=d["x"].dtype, device=DEV).transpose(1, 2)
    y, st = m.mamba_conv1d_fwd_strided(channel_major(d["x"]), d["conv_w"], d["conv_bias"], to_dev(st0), y=y_cm)
    assert_close(values(to_host(y.contiguous())), ry, TOL[io], "channel-major conv y")
    assert np.array_equal(values(to_host(st)), rst)
    assert torch.equal(y.contiguous(), y_ref) and torch.equal(st, st_ref)
    wide = torch.cat([d["x"], d["x"]], dim=2)
    y2, st2 = m.mamba_conv1d_fwd_strided(wide[..., D:], d["conv_w"], d["conv_bias"], to_dev(st0))
    assert torch.equal(y2, y_ref) and torch.equal(st2, st_ref)
    # no carried window, no activation, no state wanted
    y3, none = m.mamba_conv1d_fwd_strided(channel_major(d["x"]), d["conv_w"], None, apply_silu=False, want_state=False)
    ry3, _ = oracle.conv1d_fwd(W(c["x"]), W(c["conv_w"]), None, None, False)
    assert none is None
    assert_close(values(to_host(y3)), ry3, TOL[io], "plain conv y")


@pytest.mark.parametrize("B,L,D,kind", [(1, 1100, 576, "lanes"), (56, 130, 256, "direct"), (1, 3000, 256, "chunked")])
def test_scan_nan_stays_in_its_channel(m, B, L, D, kind):
    """A NaN in x at one (row, token, channel): that channel's outputs are NaN from that token on, and its final
    state; every other element is bit for bit what it is without the NaN (channels are independent recurrences, in
    every kernel family: across time chunks, across the lanes that scan time, across the lanes that share a channel)."""
    say(B=B, L=L, D=D, kind=kind)
    N, io = 16, synth.BF16
    assert m.mamba_scan_kernel(B, L, D, N) == kind
    c = synth.prefill_case(B, L, D, N, 4, io, seed=81000 + L)
    clean_out, clean_h = run_scan(m, c)
    b, t, d = B // 2, L // 3, D // 2 + 1
    c2 = dict(c)
    c2["x"] = c["x"].copy()
    c2["x"][b, t, d] = 0x7FC0                       # bfloat16 quiet NaN
    out, hf = run_scan(m, c2)
    o, h = values(out), hf
    assert np.isnan(o[b, t:, d]).all() and np.isnan(h[b, d]).all()
    o_mask = np.ones(o.shape, bool)
    o_mask[b, t:, d] = False
    h_mask = np.ones(h.shape, bool)
    h_mask[b, d] = False
    assert np.array_equal(out[o_mask], clean_out[o_mask]) and np.array_equal(hf[h_mask], clean_h[h_mask])
    assert not np.isnan(o[o_mask]).any()


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
def test_scan_optional_arguments(m, io):
    c = synth.prefill_case(2, 200, 128, 16, 4, io, seed=42)
    h0 = np.random.default_rng(3).standard_normal((2, 128, 16)).astype(np.float32)
    check_scan(m, c, h0=h0, z=None, what="no gate")
    check_scan(m, c, Dskip=None, what="no skip")
    check_scan(m, c, dt_bias=None, what="no dt_bias")
    c3 = dict(c)
    c3["dt"] = synth.to_io(np.abs(synth.io_values(c["dt"], io)) + 0.01, io)
    c3["dt_bias"] = np.abs(c["dt_bias"]) * 0.01
    check_scan(m, c3, h0=h0, dt_softplus=False, chunk_len=64, what="delta given directly")
    c4 = dict(c)
    c4["A"] = np.zeros_like(c["A"])
    check_scan(m, c4, h0=h0, chunk_len=32, what="A = 0")
    # no state requested
    d = dev_case(c)
    out, hf = m.mamba_scan_fwd(d["x"], d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"],
                               d["dt_bias"], want_state=False)
    assert hf is None
    ro, _ = oracle_scan(c)
    assert_close(values(to_host(out)), ro, TOL[io], "want_state=False")


def test_scan_delta_to_zero_keeps_state(m):
    # dt = -1e4 under softplus: delta underflows to 0, the state must come back bit for bit
    c = synth.prefill_case(1, 40, 64, 16, 4, synth.F32, seed=9)
    c["dt"] = np.full_like(c["dt"], -1e4)
    h0 = np.random.default_rng(1).standard_normal((1, 64, 16)).astype(np.float32)
    for cl in (0, 16):
        _, hf = run_scan(m, c, h0=h0, chunk_len=cl)
        assert np.array_equal(hf, h0)


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
def test_scan_carry_in_place_state_and_empty(m, io):
    c = synth.prefill_case(2, 300, 64, 16, 4, io, seed=11)
    d = dev_case(c)
    full, hf = m.mamba_scan_fwd(d["x"], d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"],
                                chunk_len=300)
    cut = lambda k, a, b: d[k][:, a:b].contiguous()
    state = torch.zeros((2, 64, 16), dtype=torch.float32, device=DEV)
    outs = []
    for a, b in ((0, 130), (130, 130), (130, 300)):      # the middle piece is empty
        o, _ = m.mamba_scan_fwd(cut("x", a, b), cut("dt", a, b), d["A"], cut("Bm", a, b), cut("Cm", a, b),
                                d["Dskip"], cut("z", a, b), d["dt_bias"], h0=state, h_final=state,
                                chunk_len=64)
        outs.append(o)
    tol = TOL[io]
    ro, rh = oracle_scan(c)
    assert_close(values(to_host(torch.cat(outs, 1))), ro, tol, "pieces out")
    assert_close(to_host(state), rh, tol, "pieces state")
    assert_close(to_host(hf), rh, tol, "full state")
    # empty sequence into a fresh buffer copies h0
    o, h2 = m.mamba_scan_fwd(cut("x", 0, 0), cut("dt", 0, 0), d["A"], cut("Bm", 0, 0), cut("Cm", 0, 0),
                             d["Dskip"], cut("z", 0, 0), d["dt_bias"], h0=state)
    assert torch.equal(h2, state) and o.shape[1] == 0


def test_scan_is_deterministic(m):
    c = synth.prefill_case(1, 2048, 256, 16, 4, synth.BF16, seed=5)
    a = run_scan(m, c, chunk_len=128)
    b = run_scan(m, c, chunk_len=128)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("B,L,D,kind", [(1, 1500, 576, "lanes"), (56, 200, 256, "direct"), (1, 3000, 256, "chunked")])
def test_scan_kernel_families_repeat_and_carry(m, B, L, D, kind):
    """Each kernel family as the library chooses it: two runs give the same bits; a sequence scanned in two pieces
    with the state carried over (the second piece in place on the state buffer) matches the oracle on the whole,
    whichever kernels the pieces take."""
    say(B=B, L=L, D=D, kind=kind)
    N, io = 16, synth.BF16
    assert m.mamba_scan_kernel(B, L, D, N) == kind
    c = synth.prefill_case(B, L, D, N, 4, io, seed=83000 + L, random_A=True)
    a, b = run_scan(m, c), run_scan(m, c)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    ro, rh = oracle_scan(c)
    d = dev_case(c)
    cut = 2 * L // 3 + 1
    piece = lambda k, lo, hi: d[k][:, lo:hi].contiguous()
    state = torch.zeros((B, D, N), dtype=torch.float32, device=DEV)
    outs = []
    for lo, hi in ((0, cut), (cut, L)):
        say(piece=(lo, hi), kernel=m.mamba_scan_kernel(B, hi - lo, D, N))
        o, _ = m.mamba_scan_fwd(piece("x", lo, hi), piece("dt", lo, hi), d["A"], piece("Bm", lo, hi), piece("Cm", lo, hi),
                                d["Dskip"], piece("z", lo, hi), d["dt_bias"], h0=state, h_final=state)
        outs.append(o)
    assert_close(values(to_host(torch.cat(outs, 1))), ro, TOL[io], "two pieces out")
    assert_close(to_host(state), rh, TOL[io], "two pieces state")


# ------------------------------------------------------------------------------------ step
def tok_slice(c, t):
    return {k: np.ascontiguousarray(c[k][:, t]) for k in ("x", "dt", "z", "Bm", "Cm")}


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
def test_scan_equals_repeated_steps(m, io):
    B, L, D, N = 3, 40, 128, 16
    c = synth.prefill_case(B, L, D, N, 4, io, seed=21)
    d = dev_case(c)
    h = torch.zeros((B, D, N), dtype=torch.float32, device=DEV)
    outs = []
    for t in range(L):
        _, o = m.mamba_state_step(h, d["x"][:, t].contiguous(), d["dt"][:, t].contiguous(), d["A"],
                                  d["Bm"][:, t].contiguous(), d["Cm"][:, t].contiguous(), d["Dskip"],
                                  d["z"][:, t].contiguous(), d["dt_bias"], h_out=h)       # in place
        outs.append(o)
    ro, rh = oracle_scan(c)
    assert_close(values(to_host(torch.stack(outs, 1))), ro, TOL[io], "steps out")
    assert_close(to_host(h), rh, TOL[io], "steps state")
    so, sh = m.mamba_scan_fwd(d["x"], d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"])
    assert_close(values(to_host(so)), ro, TOL[io], "scan out")
    assert_close(to_host(sh), rh, TOL[io], "scan state")


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("N", [4, 8, 16, 32])
@pytest.mark.parametrize("D", [1, 17, 100, 1536])
def test_step_against_oracle(m, io, N, D):
    say(io=io, N=N, D=D)
    n_in, n_out = 5, 11
    rng = np.random.default_rng(N * 100 + D)
    p = synth.layer_params(rng, D, N, 4, random_A=True)
    tok = synth.token_inputs(rng, (n_out,), D, N, io)
    h_in = rng.standard_normal((n_in, D, N)).astype(np.float32)
    parent = rng.integers(0, n_in, n_out).astype(np.int32)
    for gate, skip in ((True, True), (False, False)):
        ho, o = m.mamba_state_step(to_dev(h_in), to_dev(tok["x"]), to_dev(tok["dt"]), to_dev(p["A"]),
                                   to_dev(tok["Bm"]), to_dev(tok["Cm"]),
                                   to_dev(p["Dskip"]) if skip else None,
                                   to_dev(tok["z"]) if gate else None, to_dev(p["dt_bias"]),
                                   parent_idx=to_dev(parent))
        rh, ro = oracle.state_step(W(h_in), W(tok["x"]), W(tok["dt"]), W(p["A"]), W(tok["Bm"]), W(tok["Cm"]),
                                   W(p["Dskip"]) if skip else None, W(tok["z"]) if gate else None,
                                   W(p["dt_bias"]), parent)
        assert_close(to_host(ho), rh, TOL[io], "step h")
        assert_close(values(to_host(o)), ro, TOL[io], "step out")


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("N,D,K", [(16, 1536, 4), (4, 17, 2), (8, 100, 3), (32, 64, 4), (16, 1, 4), (16, 4096, 4)])
def test_conv_state_step_equals_conv_then_step(m, io, N, D, K):
    """One launch against the two-stage path (conv step through the parent index, then the state step), bit for
    bit, with and without gate / skip / conv bias / SiLU, a bad parent among the branches, and in place without
    a parent index; the two-stage path itself is compared with the oracle elsewhere."""
    say(io=io, N=N, D=D, K=K)
    n_in, n_out = 5, (70 if D >= 1536 else 11)
    rng = np.random.default_rng(N * 1000 + D + K)
    p = synth.layer_params(rng, D, N, K, random_A=True)
    p["conv_bias"] = rng.standard_normal(D).astype(np.float32)
    tok = synth.token_inputs(rng, (n_out,), D, N, io)
    h_in = to_dev(rng.standard_normal((n_in, D, N)).astype(np.float32))
    c_in = to_dev(synth.to_io(rng.standard_normal((n_in, D, K - 1)).astype(np.float32), io))
    parent = rng.integers(0, n_in, n_out).astype(np.int32)
    parent[3] = n_in + 2                                        # out of range: that branch becomes NaN in both paths
    par = to_dev(parent)
    g = {k: to_dev(v) for k, v in tok.items()}
    P = {k: to_dev(v) for k, v in p.items()}
    good = torch.as_tensor([j for j in range(n_out) if j != 3], device=DEV)
    for gate, skip, cbias, silu in ((True, True, True, True), (False, False, False, False), (True, False, True, False)):
        forked, _ = m.mamba_state_fork(c_in.unsqueeze(0), None, par)
        xc, cst = m.mamba_conv1d_fwd(g["x"].unsqueeze(1), P["conv_w"], P["conv_bias"] if cbias else None,
                                     conv_state_in=forked[0], apply_silu=silu)
        ho, o = m.mamba_state_step(h_in, xc.squeeze(1), g["dt"], P["A"], g["Bm"], g["Cm"], P["Dskip"] if skip else None,
                                   g["z"] if gate else None, P["dt_bias"], parent_idx=par)
        ho2, cst2, o2, xc2 = m.mamba_conv_state_step(h_in, c_in, g["x"], P["conv_w"], P["conv_bias"] if cbias else None,
                                                     g["dt"], P["A"], g["Bm"], g["Cm"], P["Dskip"] if skip else None,
                                                     g["z"] if gate else None, P["dt_bias"], parent_idx=par,
                                                     want_xc=True, apply_silu=silu)
        same = lambda a, b: to_host(a[good]).tobytes() == to_host(b[good]).tobytes()
        assert same(ho, ho2) and same(o, o2) and same(cst, cst2) and same(xc.squeeze(1), xc2)
        # the branch with the bad parent: NaN everywhere, except that its new window ends with its own input
        for t in (ho2[3], o2[3], xc2[3], cst2[3][:, :-1]):
            assert torch.isnan(t.float()).all()
        assert torch.equal(cst2[3][:, -1], g["x"][3])
    # sequential decode: no parent index, both states updated in place
    h = h_in.clone()
    c = c_in.clone()
    x5 = {k: v[:n_in].contiguous() for k, v in g.items()}
    xc, cst = m.mamba_conv1d_fwd(x5["x"].unsqueeze(1), P["conv_w"], P["conv_bias"], conv_state_in=c_in)
    ho, o = m.mamba_state_step(h_in, xc.squeeze(1), x5["dt"], P["A"], x5["Bm"], x5["Cm"], P["Dskip"], x5["z"], P["dt_bias"])
    _, _, o2, _ = m.mamba_conv_state_step(h, c, x5["x"], P["conv_w"], P["conv_bias"], x5["dt"], P["A"], x5["Bm"], x5["Cm"],
                                          P["Dskip"], x5["z"], P["dt_bias"], h_out=h, conv_state_out=c)
    assert torch.equal(h, ho) and torch.equal(c, cst) and torch.equal(o, o2)


def test_step_rejects_out_of_range_parent_without_reading(m):
    D, N = 64, 16
    rng = np.random.default_rng(0)
    p = synth.layer_params(rng, D, N, 4)
    tok = synth.token_inputs(rng, (3,), D, N, synth.F32)
    h_in = to_dev(rng.standard_normal((2, D, N)).astype(np.float32))
    parent = to_dev(np.array([1, 2, -1], dtype=np.int32))          # 2 and -1 are out of range
    ho, o = m.mamba_state_step(h_in, to_dev(tok["x"]), to_dev(tok["dt"]), to_dev(p["A"]), to_dev(tok["Bm"]),
                               to_dev(tok["Cm"]), parent_idx=parent)
    assert torch.isfinite(ho[0]).all() and torch.isfinite(o[0]).all()
    assert torch.isnan(ho[1:]).all() and torch.isnan(o[1:]).all()
    cd, sd = m.mamba_state_fork(None, h_in.unsqueeze(0), parent)
    assert cd is None and torch.equal(sd[0, 0], h_in[1])
    assert (sd[0, 1:].view(torch.int32) == -1).all()               # 0xFF fill


# ------------------------------------------------------------------------------------ seeded sweep
def _sweep_shapes(n, seed):
    """Shapes drawn from a fixed seed: lengths around the tile sizes the kernels use (powers of two
    +- 1, primes), odd and tiny channel counts, every state size, every window length."""
    rng = np.random.default_rng(seed)
    lens = [1, 2, 5, 31, 32, 33, 127, 128, 129, 191, 255, 256, 257, 383, 511, 513, 777, 1023, 1025, 1531]
    chans = [1, 2, 3, 31, 63, 64, 65, 96, 127, 128, 130, 257, 384, 500]
    out = []
    for i in range(n):
        out.append((int(rng.integers(1, 4)), int(rng.choice(lens)), int(rng.choice(chans)),
                    int(rng.choice([4, 8, 16, 32])), int(rng.choice([2, 3, 4])),
                    [synth.F32, synth.BF16][i % 2], int(rng.choice([0, 0, 1, 16, 37, 64, 200])), i))
    return out


@pytest.mark.parametrize("B,L,D,N,K,io,chunk_len,i", _sweep_shapes(28, 20250601))
def test_seeded_shape_sweep_conv_scan_step(m, B, L, D, N, K, io, chunk_len, i):
    say(B=B, L=L, D=D, N=N, K=K, io=io, chunk_len=chunk_len)
    if B * L * D > 600000:
        B = 1
    rng = np.random.default_rng(9000 + i)
    c = synth.prefill_case(B, L, D, N, K, io, seed=7000 + i, random_A=bool(i % 3 == 0))
    c["conv_bias"] = rng.standard_normal(D).astype(np.float32)
    st0 = synth.to_io(rng.standard_normal((B, D, K - 1)).astype(np.float32), io) if i % 2 else None
    check_conv(m, c, st0, apply_silu=bool(i % 4 != 3))
    h0 = rng.standard_normal((B, D, N)).astype(np.float32) if i % 3 != 1 else None
    kw = {}
    if i % 5 == 2:
        kw["z"] = None
    if i % 7 == 3:
        kw["Dskip"] = None
    check_scan(m, c, h0=h0, chunk_len=chunk_len, **kw)
    # one step for B * 3 branches forked from the B rows
    n_out = 3 * B
    tok = synth.token_inputs(rng, (n_out,), D, N, io)
    h_in = rng.standard_normal((B, D, N)).astype(np.float32)
    parent = rng.integers(0, B, n_out).astype(np.int32)
    ho, o = m.mamba_state_step(to_dev(h_in), to_dev(tok["x"]), to_dev(tok["dt"]), to_dev(c["A"]), to_dev(tok["Bm"]),
                               to_dev(tok["Cm"]), to_dev(c["Dskip"]), to_dev(tok["z"]), to_dev(c["dt_bias"]),
                               parent_idx=to_dev(parent))
    rh, ro = oracle.state_step(W(h_in), W(tok["x"]), W(tok["dt"]), W(c["A"]), W(tok["Bm"]), W(tok["Cm"]),
                               W(c["Dskip"]), W(tok["z"]), W(c["dt_bias"]), parent)
    assert_close(to_host(ho), rh, TOL[io], "step h")
    assert_close(values(to_host(o)), ro, TOL[io], "step out")


# ------------------------------------------------------------------------------------ fork
@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("D,N,K", [(1536, 16, 4), (17, 4, 2), (5, 8, 4), (100, 32, 3), (3, 4, 2)])
def test_fork_is_bit_exact(m, io, D, N, K):
    say(io=io, D=D, N=N, K=K)
    rng = np.random.default_rng(D + N + K)
    nl, n_in, n_out = 3, 6, 13
    ssm = rng.standard_normal((nl, n_in, D, N)).astype(np.float32)
    ssm.view(np.uint32)[0, 0, 0, 0] = 0x7FC12345                   # a NaN payload must survive
    conv = synth.to_io(rng.standard_normal((nl, n_in, D, K - 1)).astype(np.float32), io)
    parent = rng.integers(0, n_in, n_out).astype(np.int32)
    parent[0] = 0
    cd, sd = m.mamba_state_fork(to_dev(conv), to_dev(ssm), to_dev(parent))
    rc, rs = oracle.state_fork(conv, ssm, parent)
    assert to_host(cd).tobytes() == rc.tobytes()
    assert to_host(sd).tobytes() == rs.tobytes()
    c_only, none = m.mamba_state_fork(to_dev(conv), None, to_dev(parent))
    assert none is None and to_host(c_only).tobytes() == rc.tobytes()
    none, s_only = m.mamba_state_fork(None, to_dev(ssm), to_dev(parent))
    assert none is None and to_host(s_only).tobytes() == rs.tobytes()


def test_fork_paper_trees(m):
    # trees printed in the paper; children of node p sit at p*N_i .. p*N_i + N_i - 1
    D, N, K = 64, 16, 4
    rng = np.random.default_rng(12)
    for tree in ((3, 3, 2, 1), (3, 2, 2, 1, 1), (2, 2, 2, 1, 1, 1), (1, 1, 1, 1, 1)):
        ssm = to_dev(rng.standard_normal((2, 1, D, N)).astype(np.float32))
        conv = to_dev(synth.to_io(rng.standard_normal((2, 1, D, K - 1)).astype(np.float32), synth.BF16))
        root_s, root_c = ssm.clone(), conv.clone()
        for b_i, par in zip(oracle_tree.tree_batch_sizes(tree), oracle_tree.tree_parents(tree)):
            conv, ssm = m.mamba_state_fork(conv, ssm, to_dev(par))
            assert ssm.shape[1] == b_i and conv.shape[1] == b_i
        assert torch.equal(ssm, root_s.expand_as(ssm)) and torch.equal(conv, root_c.expand_as(conv))


# ------------------------------------------------------------------------------------ configs
def test_cfg0_conv_scan_and_256_steps(m):
    c = synth.config_prefill("cfg0")
    check_conv(m, c)
    e = check_scan(m, c)
    say(scan_err=e)
    d = dev_case(c)
    B, L, D, N = c["batch"], c["L"], c["D"], c["N"]
    h = torch.zeros((B, D, N), dtype=torch.float32, device=DEV)
    outs = []
    for t in range(L):
        _, o = m.mamba_state_step(h, d["x"][:, t].contiguous(), d["dt"][:, t].contiguous(), d["A"],
                                  d["Bm"][:, t].contiguous(), d["Cm"][:, t].contiguous(), d["Dskip"],
                                  d["z"][:, t].contiguous(), d["dt_bias"], h_out=h)
        outs.append(o)
    ro, rh = oracle_scan(c)
    assert_close(to_host(torch.stack(outs, 1)), ro, TOL[synth.F32], "256 steps out")
    assert_close(to_host(h), rh, TOL[synth.F32], "256 steps state")


def test_cfg0_chained_conv_then_scan(m):
    # conv output feeds the scan's x on both sides; each side runs its own chain
    c = synth.config_prefill("cfg0")
    d = dev_case(c)
    xc, _ = m.mamba_conv1d_fwd(d["x"], d["conv_w"], d["conv_bias"])
    out, hf = m.mamba_scan_fwd(xc, d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"])
    rxc, _ = oracle.conv1d_fwd(W(c["x"]), W(c["conv_w"]), W(c["conv_bias"]))
    ro, rh = oracle.scan_fwd(rxc, W(c["dt"]), W(c["A"]), W(c["Bm"]), W(c["Cm"]), W(c["Dskip"]), W(c["z"]),
                             W(c["dt_bias"]))
    assert_close(to_host(out), ro, TOL[synth.F32], "chain out")
    assert_close(to_host(hf), rh, TOL[synth.F32], "chain state")


def test_cfg1_prefill_bf16(m):
    c = synth.config_prefill("cfg1")
    check_conv(m, c)
    e = check_scan(m, c)
    say(scan_err=e)


def test_cfg3_long_prefill_every_channel(m):
    # full size on the GPU in the chunking the library picks, and the oracle on every channel of it
    c = synth.config_prefill("cfg3")
    y, st = run_conv(m, c)
    ry, rst = oracle.conv1d_fwd(W(c["x"]), W(c["conv_w"]), W(c["conv_bias"]))
    assert ry.shape == (c["batch"], c["L"], c["D"])
    assert_close(values(y), ry, TOL[c["io"]], "cfg3 conv")
    assert np.array_equal(values(st), rst)
    del y, ry
    out, hf = run_scan(m, c)
    ro, rh = oracle_scan(c)
    assert ro.shape == (c["batch"], c["L"], c["D"]) and rh.shape == (c["batch"], c["D"], c["N"])
    e1 = assert_close(values(out), ro, TOL[c["io"]], "cfg3 scan out")
    e2 = assert_close(hf, rh, TOL[c["io"]], "cfg3 scan state")
    say(scan_err=(e1, e2))
    assert m.mamba_scan_kernel(c["batch"], c["L"], c["D"], c["N"]) == "chunked"


def decode_chain_gpu(m, dc, fused):
    """fork -> conv step -> state step for every layer and draft step; returns final states and
    all step outputs.  fused: False (three stages), True (the SSM gather inside the step), "all" (one launch
    per layer: mamba_conv_state_step)."""
    nl, nb = dc["n_layers"], dc["branches"]
    ssm = to_dev(dc["ssm0"])
    conv = to_dev(dc["conv0"])
    P = [{k: to_dev(v) for k, v in p.items()} for p in dc["params"]]
    outs = []
    for s in range(dc["steps"]):
        par = to_dev(dc["parents"][s])
        if fused == "all":
            conv_next, ssm_next = torch.empty_like(conv), torch.empty_like(ssm)
            for l in range(nl):
                tok = {k: to_dev(v) for k, v in dc["tokens"][s][l].items()}
                _, _, o, _ = m.mamba_conv_state_step(ssm[l], conv[l], tok["x"], P[l]["conv_w"], P[l]["conv_bias"],
                                                     tok["dt"], P[l]["A"], tok["Bm"], tok["Cm"], P[l]["Dskip"], tok["z"],
                                                     P[l]["dt_bias"], parent_idx=par, h_out=ssm_next[l],
                                                     conv_state_out=conv_next[l])
                outs.append(o)
            conv, ssm = conv_next, ssm_next
            continue
        if fused:
            conv, _ = m.mamba_state_fork(conv, None, par)
            ssm_next = torch.empty_like(ssm)
        else:
            conv, ssm = m.mamba_state_fork(conv, ssm, par)
        for l in range(nl):
            tok = {k: to_dev(v) for k, v in dc["tokens"][s][l].items()}
            xc, _ = m.mamba_conv1d_fwd(tok["x"].unsqueeze(1), P[l]["conv_w"], P[l]["conv_bias"],
                                       conv_state_in=conv[l], conv_state_out=conv[l])
            xc = xc.squeeze(1)
            if fused:
                _, o = m.mamba_state_step(ssm[l], xc, tok["dt"], P[l]["A"], tok["Bm"], tok["Cm"],
                                          P[l]["Dskip"], tok["z"], P[l]["dt_bias"], parent_idx=par,
                                          h_out=ssm_next[l])
            else:
                _, o = m.mamba_state_step(ssm[l], xc, tok["dt"], P[l]["A"], tok["Bm"], tok["Cm"],
                                          P[l]["Dskip"], tok["z"], P[l]["dt_bias"], h_out=ssm[l])
            outs.append(o)
        if fused:
            ssm = ssm_next
    return conv, ssm, torch.stack(outs)


def decode_chain_oracle(dc, layers):
    io = dc["io"]
    ssm = dc["ssm0"][layers].astype(np.float64)
    conv = dc["conv0"][layers]
    outs = []
    for s in range(dc["steps"]):
        par = dc["parents"][s]
        conv, ssm = oracle.state_fork(conv, ssm, par)
        conv = conv.copy()
        for i, l in enumerate(layers):
            p, tok = dc["params"][l], dc["tokens"][s][l]
            xc, cst = oracle.conv1d_fwd(W(tok["x"])[:, None, :], W(p["conv_w"]), W(p["conv_bias"]), W(conv[i]))
            conv[i] = synth.to_io(cst.astype(np.float32), io)          # exact: copies of inputs
            xc_io = W(synth.to_io(xc[:, 0].astype(np.float32), io))    # the next stage reads the I/O dtype
            ssm[i], o = oracle.state_step(ssm[i], xc_io, W(tok["dt"]), W(p["A"]), W(tok["Bm"]), W(tok["Cm"]),
                                          W(p["Dskip"]), W(tok["z"]), W(p["dt_bias"]))
            outs.append(o)
    return conv, ssm, outs


def test_cfg2_tree_decode_fused_and_unfused(m):
    dc = synth.config_decode("cfg2")
    say(layers=dc["n_layers"], branches=dc["branches"], steps=dc["steps"])
    conv_u, ssm_u, out_u = decode_chain_gpu(m, dc, fused=False)
    conv_f, ssm_f, out_f = decode_chain_gpu(m, dc, fused=True)
    # fusing the gather into the step changes no bit
    assert torch.equal(ssm_u, ssm_f) and torch.equal(conv_u, conv_f) and torch.equal(out_u, out_f)
    # nor does doing fork, conv step and state update of a layer in one launch
    conv_a, ssm_a, out_a = decode_chain_gpu(m, dc, fused="all")
    assert torch.equal(ssm_u, ssm_a) and torch.equal(conv_u, conv_a) and torch.equal(out_u, out_a)
    layers = list(range(dc["n_layers"]))            # every layer of the drafter
    rconv, rssm, routs = decode_chain_oracle(dc, layers)
    nl = dc["n_layers"]
    tol = TOL[dc["io"]]
    for i, l in enumerate(layers):
        assert to_host(conv_u[l]).tobytes() == rconv[i].tobytes()
        assert_close(to_host(ssm_u[l]), rssm[i], tol, "cfg2 ssm layer %d" % l)
        for s in range(dc["steps"]):
            assert_close(values(to_host(out_u[s * nl + l])), routs[s * len(layers) + i], tol,
                         "cfg2 out step %d layer %d" % (s, l))


def test_cfg4_wide_prefill_and_decode_every_channel(m):
    cfg = synth.CONFIGS["cfg4"]
    B, L, D, N, K = cfg["batch"], cfg["L"], cfg["D"], cfg["N"], cfg["K"]
    say(B=B, L=L, D=D)
    c = synth.config_prefill("cfg4")
    d = dev_case(c)
    y, st = m.mamba_conv1d_fwd(d["x"], d["conv_w"], d["conv_bias"])
    y, st = to_host(y), to_host(st)
    out, hf = m.mamba_scan_fwd(d["x"], d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"])
    out, hf = to_host(out), to_host(hf)
    del d
    torch.cuda.empty_cache()
    # the oracle walks every channel of all 8 batch rows, a slab of channels at a time (host memory); the
    # tolerance rule's rms is the slab's: channels are identically distributed, so it is the tensor's to three digits
    slab = 512
    errs = []
    covered = np.zeros(D, dtype=bool)
    for d0 in range(0, D, slab):
        idx = np.arange(d0, min(d0 + slab, D))
        ry, rst = oracle.conv1d_fwd(W(c["x"][..., idx]), W(c["conv_w"][idx]), W(c["conv_bias"][idx]))
        assert ry.shape == (B, L, idx.size)
        assert_close(values(y[..., idx]), ry, TOL[c["io"]], "cfg4 conv, channels from %d" % d0)
        assert np.array_equal(values(st[:, idx]), rst)
        del ry
        ro, rh = oracle_scan(c, channels=idx)
        assert ro.shape == (B, L, idx.size) and rh.shape == (B, idx.size, N)
        errs.append((assert_close(values(out[..., idx]), ro, TOL[c["io"]], "cfg4 scan out, channels from %d" % d0),
                     assert_close(hf[:, idx], rh, TOL[c["io"]], "cfg4 scan state, channels from %d" % d0)))
        del ro
        covered[idx] = True
        print("    slab %d done" % d0, flush=True)
    assert covered.all()
    say(scan_err=tuple(max(e[i] for e in errs) for i in (0, 1)))
    del out, y, c
    dc = synth.config_decode("cfg4", n_layers=1)
    conv_u, ssm_u, out_u = decode_chain_gpu(m, dc, fused=False)
    conv_f, ssm_f, out_f = decode_chain_gpu(m, dc, fused=True)
    assert torch.equal(ssm_u, ssm_f) and torch.equal(out_u, out_f)
    rconv, rssm, routs = decode_chain_oracle(dc, [0])
    assert to_host(conv_u[0]).tobytes() == rconv[0].tobytes()
    assert_close(to_host(ssm_u[0]), rssm[0], TOL[dc["io"]], "cfg4 decode ssm")
    for s in range(dc["steps"]):
        assert_close(values(to_host(out_u[s])), routs[s], TOL[dc["io"]], "cfg4 decode out %d" % s)


# ------------------------------------------------------------------------------------ HIP graph
@pytest.mark.parametrize("one_launch", [False, True])
def test_decode_loop_replays_in_a_hip_graph(m, one_launch):
    """Every call has a fixed shape and neither allocates nor synchronizes, so a draft round can
    be captured once and replayed (Sec. 4.1: graph cache per batch size).  Each replay, with other
    work and synchronizations in between, must equal the eager result bit for bit."""
    dc = synth.decode_case(3, 8, 3, 256, 16, 4, synth.BF16, seed=77)
    nl, nb, D, N = dc["n_layers"], dc["branches"], dc["D"], dc["N"]
    P = [{k: to_dev(v) for k, v in p.items()} for p in dc["params"]]
    TOK = [[{k: to_dev(v) for k, v in t.items()} for t in layer] for layer in dc["tokens"]]
    PAR = [to_dev(p) for p in dc["parents"]]
    ssm0, conv0 = to_dev(dc["ssm0"]), to_dev(dc["conv0"])
    ssm = [torch.empty_like(ssm0), torch.empty_like(ssm0)]
    conv = [torch.empty_like(conv0), torch.empty_like(conv0)]
    xc = torch.empty((nb, 1, D), dtype=conv0.dtype, device=DEV)
    outs = torch.empty((dc["steps"], nl, nb, D), dtype=conv0.dtype, device=DEV)

    def draft_round():
        src_s, src_c = ssm0, conv0
        for s in range(dc["steps"]):
            dst_s, dst_c = ssm[s & 1], conv[s & 1]
            if not one_launch:
                m.mamba_state_fork(src_c, None, PAR[s], conv_dst=dst_c)
            for l in range(nl):
                t = TOK[s][l]
                if one_launch:
                    m.mamba_conv_state_step(src_s[l], src_c[l], t["x"], P[l]["conv_w"], P[l]["conv_bias"], t["dt"],
                                            P[l]["A"], t["Bm"], t["Cm"], P[l]["Dskip"], t["z"], P[l]["dt_bias"],
                                            parent_idx=PAR[s], h_out=dst_s[l], conv_state_out=dst_c[l], out=outs[s, l])
                    continue
                m.mamba_conv1d_fwd(t["x"].unsqueeze(1), P[l]["conv_w"], P[l]["conv_bias"],
                                   conv_state_in=dst_c[l], y=xc, conv_state_out=dst_c[l])
                m.mamba_state_step(src_s[l], xc.squeeze(1), t["dt"], P[l]["A"], t["Bm"], t["Cm"],
                                   P[l]["Dskip"], t["z"], P[l]["dt_bias"], parent_idx=PAR[s],
                                   h_out=dst_s[l], out=outs[s, l])
            src_s, src_c = dst_s, dst_c
        return src_s, src_c

    fin_s, fin_c = draft_round()
    torch.cuda.synchronize()
    ref = (outs.clone(), fin_s.clone(), fin_c.clone())
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            draft_round()
    torch.cuda.current_stream().wait_stream(side)
    scratch = torch.empty(1 << 22, device=DEV)
    for i in range(4):
        outs.zero_()
        ssm[0].fill_(float(i))
        ssm[1].fill_(-1.0)
        scratch.normal_()                       # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(outs, ref[0]) and torch.equal(fin_s, ref[1]) and torch.equal(fin_c, ref[2]), i


@pytest.mark.parametrize("B,L,D,kind,static", [(1, 1100, 576, "lanes", False), (56, 130, 256, "direct", False),
                                               (1, 3000, 256, "chunked", False), (1, 3000, 256, "chunked", True)])
def test_prefill_replays_in_a_hip_graph(m, B, L, D, kind, static):
    """Conv1d and scan of a prefix, every scan kernel family, captured once and replayed on new inputs written into
    the captured buffers, with other work and synchronizations in between: each replay equals the eager call on
    the same inputs bit for bit.  (The chunked family also through the entry point that brings its own chunk-state
    buffer, the one meant for callers that capture.)"""
    say(B=B, L=L, D=D, kind=kind, static=static)
    N, K, io = 16, 4, synth.BF16
    assert m.mamba_scan_kernel(B, L, D, N) == kind
    cases = [synth.prefill_case(B, L, D, N, K, io, seed=70000 + i) for i in range(3)]
    d = dev_case(cases[0])
    h0 = torch.zeros((B, D, N), dtype=torch.float32, device=DEV)
    xc, cst = torch.empty_like(d["x"]), torch.empty((B, D, K - 1), dtype=d["x"].dtype, device=DEV)
    out, hf = torch.empty_like(d["x"]), torch.empty((B, D, N), dtype=torch.float32, device=DEV)
    ws = torch.empty(max(m.mamba_scan_workspace_bytes(B, L, D, N), 16), dtype=torch.uint8, device=DEV)

    def prefill():
        m.mamba_conv1d_fwd(d["x"], d["conv_w"], d["conv_bias"], y=xc, conv_state_out=cst)
        if static:
            m.mamba_scan_fwd_static(xc, d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"], h0, out, hf)
        else:
            m.mamba_scan_fwd(xc, d["dt"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["z"], d["dt_bias"], h0=h0, out=out,
                             h_final=hf, workspace=ws)

    prefill()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            prefill()
    torch.cuda.current_stream().wait_stream(side)
    scratch = torch.empty(1 << 22, device=DEV)
    for i in (1, 2, 0, 1):
        for k in ("x", "dt", "z", "Bm", "Cm"):
            d[k].copy_(to_dev(cases[i][k]))
        h0.fill_(0.25 * i)
        prefill()                                   # eager, same buffers
        torch.cuda.synchronize()
        ref = (xc.clone(), cst.clone(), out.clone(), hf.clone())
        for t in (xc, cst, out, hf, ws):
            t.zero_()
        scratch.normal_()                           # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xc, ref[0]) and torch.equal(cst, ref[1]) and torch.equal(out, ref[2]) and torch.equal(hf, ref[3]), i
    # and against the oracle once, on the last inputs
    ro, rh = oracle.scan_fwd(values(to_host(xc)), W(cases[1]["dt"]), W(cases[0]["A"]), W(cases[1]["Bm"]), W(cases[1]["Cm"]),
                             W(cases[0]["Dskip"]), W(cases[1]["z"]), W(cases[0]["dt_bias"]),   # parameters stay those of case 0
                             np.full((B, D, N), 0.25, dtype=np.float64))
    assert_close(values(to_host(out)), ro, TOL[io], "replayed scan out")
    assert_close(to_host(hf), rh, TOL[io], "replayed scan state")


def test_softplus_and_silu_accuracy_through_the_step(m):
    """N = 4, A = 0, zero state, B = (1,0,0,0), C = (1,0,0,0), x = 1, no skip: out = delta * silu(z)
    and h[.,0] = delta, so the kernel's softplus and SiLU can be read off directly."""
    v = np.concatenate([np.linspace(-30, 30, 4001), [-80.0, -19.99, 19.99, 20.01, 50.0, 87.0]]).astype(np.float32)
    D = v.size
    one = np.zeros((1, 4), dtype=np.float32)
    one[0, 0] = 1.0
    zz = np.linspace(-25, 25, D).astype(np.float32)
    for gate in (False, True):
        ho, o = m.mamba_state_step(to_dev(np.zeros((1, D, 4), np.float32)), to_dev(np.ones((1, D), np.float32)),
                                   to_dev(v[None, :] - np.float32(0.25)), to_dev(np.zeros((D, 4), np.float32)),
                                   to_dev(one), to_dev(one), None, to_dev(zz[None, :]) if gate else None,
                                   to_dev(np.full(D, 0.25, np.float32)))
        arg = (v - np.float32(0.25)).astype(np.float64) + 0.25
        ref = np.logaddexp(0.0, arg)
        got = to_host(ho)[0, :, 0].astype(np.float64)
        rel = np.abs(got - ref) / ref
        # 3e-6: the float32 product v * log2(e) loses ~|v| * 6e-8 in the exponent at the far ends
        assert rel.max() < 3e-6, (float(rel.max()), float(arg[rel.argmax()]))
        if gate:
            z64 = zz.astype(np.float64)
            refo = ref * z64 / (1.0 + np.exp(-z64))
            goto = to_host(o)[0].astype(np.float64)
            # the exp2 arguments carry ~|z| * 6e-8 and ~|v| * 6e-8 of rounding: 1e-5 covers both factors
            assert np.all(np.abs(goto - refo) <= 1e-5 * np.abs(refo) + 1e-37)


# ------------------------------------------------------------------------------------ size limits
def test_largest_grids(m):
    """Shapes that sit on the launch-grid limits: 65535 branches / batch rows / layers, and a
    sequence long enough that the conv tiles must grow to stay within 65535 time tiles."""
    rng = np.random.default_rng(2024)
    # step: 65535 branches, tiny layer
    nb, D, N = 65535, 4, 4
    p = synth.layer_params(rng, D, N, 4, random_A=True)
    tok = synth.token_inputs(rng, (nb,), D, N, synth.F32)
    h_in = rng.standard_normal((7, D, N)).astype(np.float32)
    parent = rng.integers(0, 7, nb).astype(np.int32)
    ho, o = m.mamba_state_step(to_dev(h_in), to_dev(tok["x"]), to_dev(tok["dt"]), to_dev(p["A"]),
                               to_dev(tok["Bm"]), to_dev(tok["Cm"]), to_dev(p["Dskip"]), to_dev(tok["z"]),
                               to_dev(p["dt_bias"]), parent_idx=to_dev(parent))
    rh, ro = oracle.state_step(W(h_in), W(tok["x"]), W(tok["dt"]), W(p["A"]), W(tok["Bm"]), W(tok["Cm"]),
                               W(p["Dskip"]), W(tok["z"]), W(p["dt_bias"]), parent)
    assert_close(to_host(ho), rh, TOL[synth.F32], "65535-branch step h")
    assert_close(to_host(o), ro, TOL[synth.F32], "65535-branch step out")
    # fork: 65535 branches x 3 layers, and 65535 layers x 2 branches
    for nl, n_in, n_out in ((3, 5, 65535), (65535, 3, 2)):
        ssm = rng.standard_normal((nl, n_in, 2, 4)).astype(np.float32)
        conv = synth.to_io(rng.standard_normal((nl, n_in, 2, 3)).astype(np.float32), synth.BF16)
        par = rng.integers(0, n_in, n_out).astype(np.int32)
        cd, sd = m.mamba_state_fork(to_dev(conv), to_dev(ssm), to_dev(par))
        rc, rs = oracle.state_fork(conv, ssm, par)
        assert to_host(cd).tobytes() == rc.tobytes() and to_host(sd).tobytes() == rs.tobytes()
    # scan and conv: 65535 batch rows of a tiny layer
    c = synth.prefill_case(65535, 5, 2, 4, 3, synth.F32, seed=3)
    check_scan(m, c, what="65535-row scan")
    check_conv(m, c)
    # the single-pass kernel on as many batch rows as the grid allows
    c = synth.prefill_case(65535, 3, 8, 16, 4, synth.BF16, seed=6, random_A=True)
    assert m.mamba_scan_kernel(65535, 3, 8, 16) == "direct"
    check_scan(m, c, what="65535-row single-pass scan")
    # the scan over the lanes of a wavefront at the longest sequence it is chosen for (20 super-steps, ragged)
    assert m.mamba_scan_kernel(1, 9999, 1536, 16) == "lanes" and m.mamba_scan_kernel(1, 12000, 1536, 16) == "chunked"
    c = synth.prefill_case(1, 9999, 1536, 16, 4, synth.BF16, seed=7)
    ch = np.arange(0, 1536, 7)
    out, hf = run_scan(m, c)
    ro, rh = oracle_scan(c, channels=ch)
    assert_close(values(out)[..., ch], ro, TOL[synth.BF16], "9999-token lanes scan out")
    assert_close(hf[:, ch], rh, TOL[synth.BF16], "9999-token lanes scan state")
    # scan: as many time chunks as the grid allows (one token per chunk)
    c = synth.prefill_case(1, 65535, 2, 4, 2, synth.BF16, seed=4, random_A=True)
    check_scan(m, c, chunk_len=1, what="65535-chunk scan")
    # conv: 2.2 M tokens, more than 65535 tiles of the default length
    L = 65535 * 32 + 12345
    c = synth.prefill_case(1, L, 8, 4, 4, synth.BF16, seed=5)
    y, st = run_conv(m, c)
    idx = np.concatenate([np.arange(0, 5000), np.arange(L - 5000, L)])
    ry, rst = oracle.conv1d_fwd(W(c["x"]), W(c["conv_w"]), W(c["conv_bias"]))
    assert_close(values(y)[:, idx], ry[:, idx], TOL[synth.BF16], "2.2M-token conv (ends)")
    step = np.arange(0, L, 997)
    assert_close(values(y)[:, step], ry[:, step], TOL[synth.BF16], "2.2M-token conv (strided)")
    assert np.array_equal(values(st), rst)


def test_unsupported_sizes_are_rejected_on_the_gpu_box_too(m):
    x = torch.zeros((1, 4, 8), device=DEV)
    with pytest.raises(m.MambaError) as e:
        m.mamba_scan_fwd(x, x, torch.zeros((8, 12), device=DEV), torch.zeros((1, 4, 12), device=DEV),
                         torch.zeros((1, 4, 12), device=DEV))
    assert e.value.status == m.STATUS["UNSUPPORTED"]
    with pytest.raises(m.MambaError) as e:
        m.mamba_conv1d_fwd(x, torch.zeros((8, 5), device=DEV))
    assert e.value.status == m.STATUS["UNSUPPORTED"]
    with pytest.raises(m.MambaError) as e:                      # out aliases x
        m.mamba_conv1d_fwd(x, torch.zeros((8, 4), device=DEV), y=x)
    assert e.value.status == m.STATUS["ALIAS"]


# ------------------------------------------------------------------------------------ tree caches
@pytest.mark.parametrize("tree", [(3, 2, 2, 1, 1), (3, 3, 2, 1), (2, 2, 2, 1, 1, 1), (1, 1, 1, 1, 1), (1, 4, 1)])
def test_tree_draft_cache_against_oracle(m, tree):
    """Per-batch-size state caches + one captured graph per draft position (Sec. 4.1) on the trees the
    paper prints: every position's outputs and the final states against the oracle chain
    (fork by parent[j] = j // N_i, conv step, state step)."""
    from paper_2506_01206_amd.tree import TreeDraftCache
    say(tree=tree)
    nl, D, N, K, io = 2, 128, 16, 4, synth.BF16
    rng = np.random.default_rng(sum(tree) * 7 + len(tree))
    params = [synth.layer_params(rng, D, N, K, random_A=True) for _ in range(nl)]
    P = [{k: to_dev(v) for k, v in p.items()} for p in params]
    ssm_root = rng.standard_normal((nl, 1, D, N)).astype(np.float32)
    conv_root = synth.to_io(rng.standard_normal((nl, 1, D, K - 1)).astype(np.float32), io)
    cache = TreeDraftCache(tree, nl, D, N, K, torch.bfloat16, DEV)
    sizes = oracle_tree.tree_batch_sizes(tree)
    parents = oracle_tree.tree_parents(tree)
    assert cache.batch == [1] + sizes
    assert len(cache.ssm) == len(set([1] + sizes))                    # one cache per distinct batch size
    toks = []
    for i, b_i in enumerate(sizes, start=1):
        if tree[i - 1] > 1:
            assert np.array_equal(to_host(cache.parent[i]), parents[i - 1])
        else:
            assert cache.parent[i] is None
        layer_toks = [synth.token_inputs(rng, (b_i,), D, N, io) for _ in range(nl)]
        toks.append(layer_toks)
        for l in range(nl):
            for k in ("x", "dt", "z", "Bm", "Cm"):
                cache.inputs[i][k][l].copy_(to_dev(layer_toks[l][k]))

    def run(use_graphs):
        cache.set_root(to_dev(conv_root), to_dev(ssm_root))
        cache.draft(P, use_graphs=use_graphs)
        torch.cuda.synchronize()
        last = cache.cache_index(cache.gamma)
        return ([o.clone() for o in cache.out[1:]], cache.ssm[last].clone(), cache.conv[last].clone())

    eager = run(False)
    for _ in range(3):                                                # capture on first use, then replays
        again = run(True)
        assert all(torch.equal(a, b) for a, b in zip(eager[0], again[0]))
        assert torch.equal(eager[1], again[1]) and torch.equal(eager[2], again[2])

    ssm, conv = ssm_root.astype(np.float64), conv_root
    for i, b_i in enumerate(sizes, start=1):
        conv, ssm = oracle.state_fork(conv, ssm, parents[i - 1])
        conv = conv.copy()
        for l in range(nl):
            p, t = params[l], toks[i - 1][l]
            xc, cst = oracle.conv1d_fwd(W(t["x"])[:, None, :], W(p["conv_w"]), W(p["conv_bias"]), W(conv[l]))
            conv[l] = synth.to_io(cst.astype(np.float32), io)
            xc_io = W(synth.to_io(xc[:, 0].astype(np.float32), io))
            ssm[l], o = oracle.state_step(ssm[l], xc_io, W(t["dt"]), W(p["A"]), W(t["Bm"]), W(t["Cm"]),
                                          W(p["Dskip"]), W(t["z"]), W(p["dt_bias"]))
            assert_close(values(to_host(eager[0][i - 1][l])), o, TOL[io], "tree %s position %d layer %d" % (tree, i, l))
    assert_close(to_host(eager[1]), ssm, TOL[io], "tree final ssm")
    assert to_host(eager[2]).tobytes() == conv.tobytes()


# ------------------------------------------------------------------------------------ invariants
def test_scan_invariants_at_size(m):
    """Properties of the recurrence that hold at any size, checked on the GPU at a Mamba-130M layer
    shape (fp32 I/O): linear in x from a zero state, C = 0 leaves the gated skip, z = 0 gives 0."""
    B, L, D, N = 1, 4096, 1536, 16
    c = synth.prefill_case(B, L, D, N, 4, synth.F32, seed=808)
    d = dev_case(c)
    g = torch.Generator(device=DEV)
    g.manual_seed(1)
    x2 = torch.randn((B, L, D), device=DEV, generator=g)
    scan = lambda x, **kw: m.mamba_scan_fwd(x, d["dt"], d["A"], kw.get("Bm", d["Bm"]), kw.get("Cm", d["Cm"]),
                                           d["Dskip"], kw.get("z", d["z"]), d["dt_bias"])
    o1, h1 = scan(d["x"])
    o2, h2 = scan(x2)
    a, b = 0.75, -1.5
    o3, h3 = scan(a * d["x"] + b * x2)
    ref_o, ref_h = (a * o1.double() + b * o2.double()).cpu().numpy(), (a * h1.double() + b * h2.double()).cpu().numpy()
    assert_close(to_host(o3), ref_o, 1e-4, "linearity out")
    assert_close(to_host(h3), ref_h, 1e-4, "linearity state")
    o4, _ = scan(d["x"], Cm=torch.zeros_like(d["Cm"]))
    zz = d["z"].double()
    ref = (d["x"].double() * zz / (1 + torch.exp(-zz))).cpu().numpy()        # D = 1
    assert_close(to_host(o4), ref, 1e-5, "C = 0")
    o5, h5 = scan(d["x"], z=torch.zeros_like(d["z"]))
    assert torch.count_nonzero(o5) == 0 and torch.equal(h5, h1)             # the gate never touches the state


# ------------------------------------------------------------------------------------ dense parts
@pytest.mark.parametrize("M,N,K,splits", [(1, 1, 8, None), (5, 80, 48, (48, 16, 16)), (130, 200, 72, None),
                                          (257, 3072, 768, (1536, 1536)), (1000, 80, 1536, (48, 16, 16)),
                                          (384, 768, 1536, None), (64, 1536, 48, None), (129, 129, 1032, (1, 128)),
                                          # few rows (draft positions): the split-k kernel, one or two row blocks
                                          (18, 3072, 768, (1536, 1536)), (12, 80, 1536, (48, 16, 16)), (32, 768, 1536, None),
                                          (33, 100, 520, (3, 90, 7)), (64, 50, 1544, None), (3, 1000, 72, None),
                                          (65, 96, 512, None),
                                          # few rows, very wide (the LM head): tiled kernel with streaming weight loads
                                          (12, 8200, 136, None), (64, 9000, 64, (8192, 808)),
                                          # more than a thousand 128 x 128 tiles (ragged edges, short and odd slab counts)
                                          (8190, 4100, 136, (2052, 2048)), (8192, 4096, 40, None), (8300, 4000, 32, (8, 3992)),
                                          # whole slabs only (K a multiple of 64): 1, 2, 3, 5 and 7 of them, ragged edges,
                                          # split outputs
                                          (4096, 4096, 64, None), (4100, 4000, 128, (2000, 2000)), (4096, 4104, 192, None),
                                          (4090, 4096, 320, (4088, 8)), (5000, 3400, 448, (1000, 1200, 1200)),
                                          # 256-row tiles, 256 and 128 columns wide (M % 256 == 0, K % 128 == 0, >= 512 tiles):
                                          # 4, 6, 8 and 10 slabs, splits on and off the tile edges
                                          (16384, 2048, 256, (1024, 1024)), (16384, 1152, 384, None), (8192, 4096, 512, None),
                                          (16384, 1152, 640, (1000, 152)), (1024, 3072, 768, (1536, 1536)), (512, 6144, 128, None),
                                          # 128 x 128 tiles of the same kernel (M % 128 == 0, 192 .. a few hundred tiles)
                                          (4096, 768, 1536, None), (2688, 1152, 256, (1000, 152)), (384, 8192, 384, None)])
def test_linear_against_oracle(m, M, N, K, splits):
    say(M=M, N=N, K=K, splits=splits)
    rng = np.random.default_rng(M + N + K)
    x = synth.to_io(rng.standard_normal((M, K)).astype(np.float32), synth.BF16)
    w = synth.to_io((rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32), synth.BF16)
    bias = rng.standard_normal(N).astype(np.float32)
    ref = oracle.linear(W(x), W(w), W(bias))
    outs = m.mamba_linear_fwd(to_dev(x), to_dev(w), to_dev(bias), splits=splits)
    got = np.concatenate([values(to_host(o)) for o in outs], axis=1)
    assert_close(got, ref, TOL[synth.BF16], "linear")
    if splits is None:
        res = synth.to_io(rng.standard_normal((M, N)).astype(np.float32), synth.BF16)
        buf = to_dev(res)
        (o,) = m.mamba_linear_fwd(to_dev(x), to_dev(w), None, residual=buf, outs=[buf])      # in place on the residual
        assert_close(values(to_host(o)), oracle.linear(W(x), W(w), None, W(res)), TOL[synth.BF16], "linear + residual")


def test_linear_at_block_bench_size_sampled_rows(m):
    """in_proj and out_proj of the whole-block leg of bench.py (32768 tokens, Mamba-130M widths), in the launch
    configuration it times; rows are independent, so the oracle computes a seeded sample of them (every row block
    of the first and last tiles, and rows scattered over the rest)."""
    M = 32768
    rng = np.random.default_rng(321)
    rows = np.unique(np.concatenate([np.arange(0, 256, 5), np.arange(M - 256, M, 7), rng.integers(0, M, 300)]))
    for (N, K, splits, with_res) in ((3072, 768, (1536, 1536), False), (768, 1536, None, True)):
        say(M=M, N=N, K=K, splits=splits, residual=with_res, sampled_rows=len(rows))
        x = synth.to_io(rng.standard_normal((M, K)).astype(np.float32), synth.BF16)
        w = synth.to_io((rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32), synth.BF16)
        res = synth.to_io(rng.standard_normal((M, N)).astype(np.float32), synth.BF16) if with_res else None
        outs = m.mamba_linear_fwd(to_dev(x), to_dev(w), None, residual=to_dev(res), splits=splits)
        got = np.concatenate([values(to_host(o[torch.as_tensor(rows, device=DEV)])) for o in outs], axis=1)
        ref = oracle.linear(W(x[rows]), W(w), None, None if res is None else W(res[rows]))
        assert_close(got, ref, TOL[synth.BF16], "linear at bench size")


def test_linear_wide_tiles_are_deterministic(m):
    """The 256-row tiles stream their operands into LDS asynchronously and order them with explicit waits; a
    missing wait would show as run-to-run differences.  Ten launches each, all three tile shapes, on fresh outputs."""
    g = torch.Generator(device=DEV)
    g.manual_seed(77)
    for (M, N, K) in ((8192, 4096, 768), (16384, 1152, 1536), (4096, 768, 1536)):
        x = torch.randn(M, K, device=DEV, generator=g).bfloat16()
        w = (torch.randn(N, K, device=DEV, generator=g) / K ** 0.5).bfloat16()
        (first,) = m.mamba_linear_fwd(x, w)
        for _ in range(9):
            out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
            m.mamba_linear_fwd(x, w, outs=[out])
            assert torch.equal(out, first)


@pytest.mark.parametrize("M,C", [(1, 8), (7, 768), (1000, 768), (33, 2048), (5, 4096), (3, 40)])
def test_rmsnorm_against_oracle(m, M, C):
    rng = np.random.default_rng(M + C)
    x = synth.to_io((rng.standard_normal((M, C)) * rng.uniform(0.01, 30, (M, 1))).astype(np.float32), synth.BF16)
    w = rng.standard_normal(C).astype(np.float32)
    y = m.mamba_rmsnorm_fwd(to_dev(x), to_dev(w), eps=1e-5)
    assert_close(values(to_host(y)), oracle.rmsnorm(W(x), W(w), 1e-5), TOL[synth.BF16], "rmsnorm")
    xin = to_dev(x)
    m.mamba_rmsnorm_fwd(xin, to_dev(w), eps=1e-5, y=xin)                                   # in place
    assert torch.equal(xin, y)


# ------------------------------------------------------------------------------------ whole block
def make_block(m, rng, dm, D, N, K, R):
    w = synth.block_weights(rng, dm, D, N, K, R)
    dev = {k: to_dev(v) for k, v in w.items()}
    return w, {k: W(v) for k, v in w.items()}, m.Block(dev, eps=1e-5)


def check_block_stages(m, blk, w64, hid, conv_in=None, h0=None, what="block"):
    """One call of mamba_block_fwd, then every stage against the oracle of that stage fed with the tensors the
    device itself stored in front of it (read back from the workspace), each at the plain tolerance: a bf16 rounding
    flip upstream then is an input both sides share, not an error the next stage amplifies.  The first three stages
    (RMSNorm, in_proj, conv1d) are checked as a chain, since their intermediate buffers are reused later in the call.
    hid: (B,L,d_model) bf16 bits; conv_in bf16 bits or None; h0 float32 or None.  Returns the device results."""
    B, L, dm = hid.shape
    D, N = w64["A"].shape
    R = w64["dt_proj_w"].shape[1]
    tol = TOL[synth.BF16]
    ws = torch.empty(max(m.mamba_block_workspace_bytes(blk, B, L), 16), dtype=torch.uint8, device=DEV)
    out, cst, hf = m.mamba_block_fwd(blk, to_dev(hid), conv_state_in=to_dev(conv_in), h0=to_dev(h0), workspace=ws)
    torch.cuda.synchronize()
    st = {k: values(to_host(v)) for k, v in m.mamba_block_workspace_layout(blk, B, L, ws).items()}
    rb = oracle._round_bf16
    # RMSNorm -> in_proj -> conv1d + SiLU, storage roundings in between
    u = rb(oracle.rmsnorm(W(hid).reshape(B * L, dm), w64["norm_w"], 1e-5))
    xz = oracle.linear(u, w64["in_proj_w"])
    assert_close(st["z"], xz[:, D:], tol, what + ": z")
    xc, rcs = oracle.conv1d_fwd(rb(xz[:, :D]).reshape(B, L, D), w64["conv_w"], w64.get("conv_b"), W(conv_in))
    assert_close(st["x_c"], xc.reshape(B * L, D), tol, what + ": x_c")
    assert_close(values(to_host(cst)), rcs, tol, what + ": conv state")
    # x_proj on the device's x_c
    proj = oracle.linear(st["x_c"], w64["x_proj_w"])
    assert_close(np.concatenate([st["dt_low"], st["B"], st["C"]], axis=1), proj, tol, what + ": dt_low | B | C")
    # dt_proj on the device's dt_low
    assert_close(st["dt"], oracle.linear(st["dt_low"], w64["dt_proj_w"]), tol, what + ": dt")
    # selective scan on the device's x_c, dt, B, C, z
    ry, rh = oracle.scan_fwd(st["x_c"].reshape(B, L, D), st["dt"].reshape(B, L, D), w64["A"], st["B"].reshape(B, L, N),
                             st["C"].reshape(B, L, N), w64["Dskip"], st["z"].reshape(B, L, D), w64["dt_bias"],
                             None if h0 is None else h0.astype(np.float64))
    e_y = assert_close(st["y"], ry.reshape(B * L, D), tol, what + ": y")
    e_h = assert_close(to_host(hf), rh, tol, what + ": ssm state")
    # out_proj + residual on the device's y
    ro = oracle.linear(st["y"], w64["out_proj_w"], None, W(hid).reshape(B * L, dm)).reshape(B, L, dm)
    assert_close(values(to_host(out)), ro, tol, what + ": hidden out")
    say(stage_err_y=e_y, stage_err_state=e_h)
    return out, cst, hf


@pytest.mark.parametrize("B,L,dm,D,N,K,R", [(2, 96, 64, 128, 16, 4, 8), (1, 700, 768, 1536, 16, 4, 48),
                                           (3, 33, 256, 512, 8, 3, 16),
                                           # long enough for the 256-row projection tiles (in_proj and out_proj)
                                           (1, 4096, 768, 1536, 16, 4, 48),
                                           # 32 states, the fastest of them decaying by exp(-16 delta) a step
                                           (2, 100, 216, 1144, 32, 3, 24)])
def test_block_prefill_against_oracle(m, B, L, dm, D, N, K, R):
    """RMSNorm -> in_proj -> conv1d -> x_proj -> dt_proj -> selective scan -> out_proj + residual as one call:
    every stage against its oracle at the plain tolerance (check_block_stages), the whole block against the
    float64 block evaluated without any rounding in between (looser: six bf16 roundings on the way), and the
    same again in two pieces with carried conv / SSM states."""
    say(B=B, L=L, dm=dm, D=D, N=N, K=K, R=R)
    rng = np.random.default_rng(B * 1000 + L + D)
    w, w64, blk = make_block(m, rng, dm, D, N, K, R)
    hid = synth.to_io(rng.standard_normal((B, L, dm)).astype(np.float32), synth.BF16)
    out, cst, hf = check_block_stages(m, blk, w64, hid)
    tol = TOL[synth.BF16]
    ro64, _, rh64 = oracle.block_fwd(w64, W(hid), round_between=False)
    assert_close(values(to_host(out)), ro64, 3 * tol, "block out vs unrounded float64")
    # two pieces with carried states: stage by stage again, and the same result as the single call up to the tolerance
    cut = L // 3
    o1, c1, s1 = check_block_stages(m, blk, w64, hid[:, :cut], what="first piece")
    o2, c2, s2 = check_block_stages(m, blk, w64, hid[:, cut:], conv_in=to_host(c1), h0=to_host(s1), what="second piece")
    assert_close(values(to_host(torch.cat([o1, o2], 1))), ro64, 3 * tol, "block pieces out vs unrounded float64")
    assert_close(values(to_host(c2)), values(to_host(cst)), tol, "conv state, pieces vs single call")
    # in place on the residual stream
    h2 = to_dev(hid).clone()
    m.mamba_block_fwd(blk, h2, hidden_out=h2)
    assert torch.equal(h2, out)


@pytest.mark.parametrize("tree", [(3, 2, 1), (1, 1), (4,), (33, 2, 1), (66, 2)])
def test_block_decode_steps_against_oracle(m, tree):
    """Tree drafting through whole blocks: at every draft position each branch continues from its
    parent's conv and SSM state (fork fused into the step) and produces the next hidden row."""
    dm, D, N, K, R = 768, 1536, 16, 4, 48
    rng = np.random.default_rng(sum(tree) + 100)
    w, w64, blk = make_block(m, rng, dm, D, N, K, R)
    conv = synth.to_io(rng.standard_normal((1, D, K - 1)).astype(np.float32), synth.BF16)
    ssm = rng.standard_normal((1, D, N)).astype(np.float32)
    g_conv, g_ssm = to_dev(conv), to_dev(ssm)
    r_conv, r_ssm = W(conv), ssm.astype(np.float64)
    tol = TOL[synth.BF16]
    for n_i, b_i, par in zip(tree, oracle_tree.tree_batch_sizes(tree), oracle_tree.tree_parents(tree)):
        hid = synth.to_io(rng.standard_normal((b_i, dm)).astype(np.float32), synth.BF16)
        if n_i > 1:
            out, g_conv, g_ssm = m.mamba_block_step(blk, to_dev(hid), g_conv, g_ssm, parent_idx=to_dev(par))
        else:
            out, g_conv, g_ssm = m.mamba_block_step(blk, to_dev(hid), g_conv, g_ssm)       # in place
        ro, r_conv, r_ssm = oracle.block_fwd(w64, W(hid)[:, None, :], conv_state_in=r_conv[par], h0=r_ssm[par])
        assert_close(values(to_host(out)), ro[:, 0], tol, "block step out (batch %d)" % b_i)
        assert_close(to_host(g_ssm), r_ssm, tol, "block step ssm")
        assert_close(values(to_host(g_conv)), r_conv, tol, "block step conv")
        r_conv = W(synth.to_io(r_conv.astype(np.float32), synth.BF16))


@pytest.mark.parametrize("dm,D,N,K,R", [(1024, 2048, 32, 3, 64), (640, 1280, 8, 2, 40), (768, 1600, 16, 4, 48)])
def test_block_decode_steps_other_shapes(m, dm, D, N, K, R):
    """The fused draft-position chain on other layer shapes: more states and a wider low-rank dt (the x projection
    then has 128 columns), fewer states, and a d_inner whose column blocks do not come in fours, which takes the
    chain with the x projection as a launch of its own."""
    say(dm=dm, D=D, N=N, K=K, R=R)
    rng = np.random.default_rng(dm + D + N)
    w, w64, blk = make_block(m, rng, dm, D, N, K, R)
    conv = synth.to_io(rng.standard_normal((1, D, K - 1)).astype(np.float32), synth.BF16)
    ssm = rng.standard_normal((1, D, N)).astype(np.float32)
    g_conv, g_ssm = to_dev(conv), to_dev(ssm)
    r_conv, r_ssm = W(conv), ssm.astype(np.float64)
    tol = TOL[synth.BF16]
    tree = (5, 2, 1)
    for n_i, b_i, par in zip(tree, oracle_tree.tree_batch_sizes(tree), oracle_tree.tree_parents(tree)):
        hid = synth.to_io(rng.standard_normal((b_i, dm)).astype(np.float32), synth.BF16)
        if n_i > 1:
            out, g_conv, g_ssm = m.mamba_block_step(blk, to_dev(hid), g_conv, g_ssm, parent_idx=to_dev(par))
        else:
            out, g_conv, g_ssm = m.mamba_block_step(blk, to_dev(hid), g_conv, g_ssm)
        ro, r_conv, r_ssm = oracle.block_fwd(w64, W(hid)[:, None, :], conv_state_in=r_conv[par], h0=r_ssm[par])
        assert_close(values(to_host(out)), ro[:, 0], tol, "block step out (batch %d)" % b_i)
        assert_close(to_host(g_ssm), r_ssm, tol, "block step ssm")
        assert_close(values(to_host(g_conv)), r_conv, tol, "block step conv")
        r_conv = W(synth.to_io(r_conv.astype(np.float32), synth.BF16))


def test_block_step_bad_parent_poisons_only_that_branch(m):
    """A parent index outside the source cache cannot be honoured: that branch's states and hidden row
    come back NaN (never an out-of-bounds read), the other branches are untouched by it."""
    dm, D, N, K, R = 64, 128, 16, 4, 8
    rng = np.random.default_rng(77)
    w, w64, blk = make_block(m, rng, dm, D, N, K, R)
    conv = to_dev(synth.to_io(rng.standard_normal((2, D, K - 1)).astype(np.float32), synth.BF16))
    ssm = to_dev(rng.standard_normal((2, D, N)).astype(np.float32))
    hid = to_dev(synth.to_io(rng.standard_normal((3, dm)).astype(np.float32), synth.BF16))
    good = m.mamba_block_step(blk, hid, conv, ssm, parent_idx=to_dev(np.array([1, 0, 1], dtype=np.int32)))
    bad = m.mamba_block_step(blk, hid, conv, ssm, parent_idx=to_dev(np.array([1, 2, -1], dtype=np.int32)))
    for g, b in zip(good, bad):
        assert torch.equal(g[0], b[0])
    out, conv_new, ssm_new = bad
    assert torch.isnan(out[1:].float()).all() and torch.isnan(ssm_new[1:]).all()
    # the window keeps the branch's own new column; the columns inherited from the missing parent are NaN
    assert torch.isnan(conv_new[1:, :, :K - 2].float()).all() and torch.equal(conv_new[1:, :, K - 2], good[1][1:, :, K - 2])


# ------------------------------------------------------------------------------------ vocabulary ends
@pytest.mark.parametrize("M,V,k", [(1, 5, 3), (7, 1000, 8), (32, 50280, 3), (3, 257, 1), (2, 4, 8), (9, 10003, 8),
                                   (4, 20, 5)])
def test_topk_is_exact(m, M, V, k):
    rng = np.random.default_rng(M + V + k)
    x = synth.to_io(rng.standard_normal((M, V)).astype(np.float32), synth.BF16)      # bf16: many exact ties
    vals = values(x)
    idx, val = m.mamba_topk_fwd(to_dev(x), k)
    ri, rv = oracle.topk(vals, k)
    assert np.array_equal(to_host(idx), ri)                                           # integer work: bit-exact
    assert np.array_equal(to_host(val).astype(np.float64), rv)
    if V > 10:
        xn = vals.astype(np.float32).copy()
        xn[0, 1] = np.nan
        xn[0, 2] = np.inf
        i2, _ = m.mamba_topk_fwd(torch.from_numpy(xn).to(DEV).to(torch.bfloat16), k)
        assert to_host(i2)[0, 0] == 2 and 1 not in to_host(i2)[0]


def test_embedding_is_a_gather(m):
    rng = np.random.default_rng(3)
    V, dm = 1000, 768
    table = synth.to_io(rng.standard_normal((V, dm)).astype(np.float32), synth.BF16)
    tok = rng.integers(0, V, 77).astype(np.int32)
    out = m.mamba_embedding_fwd(to_dev(tok), to_dev(table))
    assert to_host(out).tobytes() == oracle.embedding(tok, table).tobytes()
    bad = m.mamba_embedding_fwd(to_dev(np.array([5, V, -1], dtype=np.int32)), to_dev(table))
    assert torch.equal(bad[0], to_dev(table)[5]) and torch.isnan(bad[1:].float()).all()


# ------------------------------------------------------------------------------------ whole drafter
def make_drafter(m, seed, V, dm, D, N, K, R, nl, L):
    rng = np.random.default_rng(seed)
    blocks = [synth.block_weights(rng, dm, D, N, K, R) for _ in range(nl)]
    emb = synth.f32_to_bf16_bits(rng.standard_normal((V, dm)).astype(np.float32))
    head = synth.f32_to_bf16_bits(rng.standard_normal((V, dm)).astype(np.float32))
    norm_f = (1 + 0.1 * rng.standard_normal(dm)).astype(np.float32)
    toks = rng.integers(0, V, L).astype(np.int32)
    w64 = dict(embedding=W(emb), lm_head=W(head), norm_f=W(norm_f), blocks=[{k: W(v) for k, v in b.items()} for b in blocks])
    from paper_2506_01206_amd.drafter import MambaDrafter
    gpu = MambaDrafter(to_dev(emb), [m.Block({k: to_dev(v) for k, v in b.items()}, eps=1e-5) for b in blocks],
                       to_dev(norm_f), lm_head=to_dev(head))
    return w64, gpu, toks


def test_drafter_tree_tokens_match_the_oracle(m):
    """Prefix encoding, then a (2, 2, 1, 1) tree drafted end to end on the device (top-N_i candidates ->
    embedding -> blocks with the state fork -> final norm -> LM head), eagerly and as one captured
    graph replayed twice.  Token choices are integer results decided by bf16 logits, so the comparison
    is exact only where the oracle's candidates are clearly separated: the seed is one where every gap
    between ranked candidates exceeds 0.15 of the logits' rms, checked first, eight times the tolerance."""
    from oracle import drafter as od
    tree = (2, 2, 1, 1)
    w64, gpu, toks = make_drafter(m, 106, V=48, dm=64, D=128, N=16, K=4, R=8, nl=2, L=40)
    lg, cs, hs = od.prefill(w64, toks)
    r_tok, r_logits, gap = od.draft(w64, tree, lg, cs, hs)
    rms = np.sqrt(np.mean(r_logits[-1] ** 2))
    assert gap > 0.15 * rms, "the seed no longer separates the candidates; pick another"
    tol = TOL[synth.BF16]
    g_lg = gpu.prefill(to_dev(toks))
    assert_close(values(to_host(g_lg)), lg, tol, "prefix logits")
    # per block: the same launches as prefill() one block at a time, every stage of block l against its oracle on
    # the hidden rows the device fed it (plain tolerance at every depth), and prefill()'s root states bit-identical
    hid_dev = m.mamba_embedding_fwd(to_dev(toks), gpu.embedding).view(1, len(toks), gpu.dm)
    for l, blk in enumerate(gpu.blocks):
        hid_bits = to_host(hid_dev)
        hid_dev, c_l, s_l = check_block_stages(m, blk, w64["blocks"][l], hid_bits, what="prefix block %d" % l)
        assert torch.equal(s_l, gpu.root_ssm[l]) and torch.equal(c_l, gpu.root_conv[l])
    for mode, use_graph in (("eager", False), ("graph capture", True), ("graph replay", True)):
        say(mode=mode)
        g_tok, g_last = gpu.draft(tree, use_graph=use_graph)
        torch.cuda.synchronize()
        for i, (gt, rt) in enumerate(zip(g_tok, r_tok)):
            assert np.array_equal(to_host(gt), rt), "%s: draft tokens at position %d" % (mode, i + 1)
        assert_close(values(to_host(g_last)), r_logits[-1], tol, mode + ": logits after the last position")
    # a second prefix through the same captured graph: the root is an input, not baked in
    toks2 = np.roll(toks, 14)
    lg2, cs2, hs2 = od.prefill(w64, toks2)
    r_tok2, r_logits2, gap2 = od.draft(w64, tree, lg2, cs2, hs2)
    assert gap2 > 0.12 * rms
    gpu.prefill(to_dev(toks2))
    g_tok2, g_last2 = gpu.draft(tree)
    torch.cuda.synchronize()
    for gt, rt in zip(g_tok2, r_tok2):
        assert np.array_equal(to_host(gt), rt)
    assert_close(values(to_host(g_last2)), r_logits2[-1], tol, "second prefix, last logits")


# ------------------------------------------------------------------------------------ Mamba-2 style core
def ssd_case(rng, B, L, H, P, N, io):
    c = dict(x=rng.standard_normal((B, L, H, P)), z=rng.standard_normal((B, L, H, P)), dt=0.5 * rng.standard_normal((B, L, H)),
             Bm=rng.standard_normal((B, L, N)), Cm=rng.standard_normal((B, L, N)))
    c = {k: synth.to_io(v.astype(np.float32), io) for k, v in c.items()}
    c.update(A=(-rng.uniform(0.05, 1.5, H)).astype(np.float32), Dskip=rng.standard_normal(H).astype(np.float32),
             dt_bias=rng.uniform(-4.0, -1.0, H).astype(np.float32), h0=rng.standard_normal((B, H, P, N)).astype(np.float32))
    return c


@pytest.mark.parametrize("B,L,H,N", [(1, 64, 2, 64), (2, 200, 3, 128), (1, 1, 1, 128), (1, 63, 2, 64), (1, 65, 2, 128),
                                     (1, 1000, 24, 128), (2, 500, 64, 64), (1, 330, 100, 128), (4, 130, 64, 64)])
def test_ssd_scan_against_oracle(m, B, L, H, N):
    """Chunked scalar-decay scan on the matrix cores against the plain float64 recurrence: outputs and final
    state, with and without gate / skip / initial state, and in two pieces with the state carried."""
    from oracle import ssd
    say(B=B, L=L, H=H, N=N)
    P = 64
    rng = np.random.default_rng(B * 7 + L + H + N)
    c = ssd_case(rng, B, L, H, P, N, synth.BF16)
    w = {k: W(v) for k, v in c.items()}
    g = {k: to_dev(v) for k, v in c.items()}
    tol = TOL[synth.BF16]
    out, hf = m.mamba2_ssd_fwd(g["x"], g["dt"], g["A"], g["Bm"], g["Cm"], g["Dskip"], g["z"], g["dt_bias"], g["h0"])
    ro, rh = ssd.ssd_scan(w["x"], w["dt"], w["A"], w["Bm"], w["Cm"], w["Dskip"], w["z"], w["dt_bias"], w["h0"])
    assert_close(values(to_host(out)), ro, tol, "ssd out")
    assert_close(to_host(hf), rh, tol, "ssd final state")
    out2, hf2 = m.mamba2_ssd_fwd(g["x"], g["dt"], g["A"], g["Bm"], g["Cm"])
    ro2, rh2 = ssd.ssd_scan(w["x"], w["dt"], w["A"], w["Bm"], w["Cm"])
    assert_close(values(to_host(out2)), ro2, tol, "ssd out, bare")
    assert_close(to_host(hf2), rh2, tol, "ssd final state, bare")
    if L > 2:
        cut = L // 3
        sl = lambda t, a, b: t[:, a:b].clone()
        o1, h1 = m.mamba2_ssd_fwd(sl(g["x"], 0, cut), sl(g["dt"], 0, cut), g["A"], sl(g["Bm"], 0, cut), sl(g["Cm"], 0, cut),
                                  g["Dskip"], sl(g["z"], 0, cut), g["dt_bias"], g["h0"])
        o2, h2 = m.mamba2_ssd_fwd(sl(g["x"], cut, L), sl(g["dt"], cut, L), g["A"], sl(g["Bm"], cut, L), sl(g["Cm"], cut, L),
                                  g["Dskip"], sl(g["z"], cut, L), g["dt_bias"], h1)
        assert_close(values(to_host(torch.cat([o1, o2], 1))), ro, tol, "ssd pieces out")
        assert_close(to_host(h2), rh, tol, "ssd pieces state")


def test_ssd_scan_at_bench_size_sampled_heads(m):
    """The scan at the size and launch configuration bench.py times (32768 tokens, 24 heads, 128 states: ten
    segments per head in the output pass, twenty in the state pass).  Heads are independent, so the oracle runs
    on two sampled heads only and is compared with the same heads of the full-size result."""
    from oracle import ssd
    B, L, H, P, N = 1, 32768, 24, 64, 128
    say(B=B, L=L, H=H, N=N)
    rng = np.random.default_rng(5)
    c = ssd_case(rng, B, L, H, P, N, synth.BF16)
    g = {k: to_dev(v) for k, v in c.items()}
    out, hf = m.mamba2_ssd_fwd(g["x"], g["dt"], g["A"], g["Bm"], g["Cm"], g["Dskip"], g["z"], g["dt_bias"], g["h0"])
    out, hf = values(to_host(out)), to_host(hf)
    tol = TOL[synth.BF16]
    w = {k: W(v) for k, v in c.items()}
    for h in (3, 23):
        ro, rh = ssd.ssd_scan(w["x"][:, :, h:h + 1], w["dt"][:, :, h:h + 1], w["A"][h:h + 1], w["Bm"], w["Cm"], w["Dskip"][h:h + 1],
                              w["z"][:, :, h:h + 1], w["dt_bias"][h:h + 1], w["h0"][:, h:h + 1])
        assert_close(out[:, :, h:h + 1], ro, tol, "ssd out, head %d" % h)
        assert_close(hf[:, h:h + 1], rh, tol, "ssd final state, head %d" % h)


@pytest.mark.parametrize("io", [synth.F32, synth.BF16])
@pytest.mark.parametrize("n_out,n_in,H,N", [(5, 3, 2, 64), (12, 6, 24, 128), (1, 1, 1, 128)])
def test_ssd_state_step_against_oracle(m, io, n_out, n_in, H, N):
    from oracle import ssd
    P = 64
    rng = np.random.default_rng(n_out + n_in + H + N)
    c = ssd_case(rng, n_out, 1, H, P, N, io)
    tok = {k: c[k][:, 0] for k in ("x", "z", "dt", "Bm", "Cm")}
    h_in = rng.standard_normal((n_in, H, P, N)).astype(np.float32)
    parent = rng.integers(0, n_in, n_out).astype(np.int32)
    g = {k: to_dev(np.ascontiguousarray(v)) for k, v in tok.items()}
    w = {k: W(np.ascontiguousarray(v)) for k, v in tok.items()}
    ho, out = m.mamba2_state_step(to_dev(h_in), g["x"], g["dt"], to_dev(c["A"]), g["Bm"], g["Cm"], to_dev(c["Dskip"]), g["z"],
                                  to_dev(c["dt_bias"]), parent_idx=to_dev(parent))
    rh, ro = ssd.ssd_step(h_in, w["x"], w["dt"], W(c["A"]), w["Bm"], w["Cm"], W(c["Dskip"]), w["z"], W(c["dt_bias"]), parent=parent)
    assert_close(values(to_host(out)), ro, TOL[io], "ssd step out")
    assert_close(to_host(ho), rh, TOL[synth.F32] if io == synth.F32 else 1e-5, "ssd step state")
    if n_in == n_out:
        hbuf = to_dev(h_in)
        m.mamba2_state_step(hbuf, g["x"], g["dt"], to_dev(c["A"]), g["Bm"], g["Cm"], h_out=hbuf)            # in place
        rh2, _ = ssd.ssd_step(h_in, w["x"], w["dt"], W(c["A"]), w["Bm"], w["Cm"])
        assert_close(to_host(hbuf), rh2, 1e-5, "ssd step in place")
    bad = parent.copy()
    bad[0] = n_in
    ho2, out2 = m.mamba2_state_step(to_dev(h_in), g["x"], g["dt"], to_dev(c["A"]), g["Bm"], g["Cm"], parent_idx=to_dev(bad))
    assert torch.isnan(ho2[0]).all() and torch.isnan(out2[0].float()).all() and not torch.isnan(ho2[1:]).any()
