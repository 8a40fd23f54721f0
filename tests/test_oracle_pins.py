"""Pins for the fp64 oracle: closed forms, invariants, library reductions, brute force.

None of these tests re-types the oracle's own loop.  Each compares it with
something fixed by the mathematics of the layer definition (the selective SSM
recurrence h_t = exp(delta_t A) h_{t-1} + delta_t B_t x_t, y_t = C_t h_t + D x_t,
gated by silu(z), delta = softplus(dt + dt_bias); depthwise causal conv1d) or by
the paper (Sec. 4.1: a child node copies its parent's state; batch size at draft
position i is N_1 x ... x N_i; the next token depends only on the current state).
"""
import os

import numpy as np
import pytest
from scipy.special import expit

import oracle
from oracle import tree as oracle_tree
from paper_2506_01206_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(seed):
    return np.random.default_rng(seed)


def rand_case(seed, B=2, L=7, D=3, N=4, with_h0=True):
    r = rnd(seed)
    c = dict(
        x=r.standard_normal((B, L, D)), dt=0.3 * r.standard_normal((B, L, D)),
        z=r.standard_normal((B, L, D)), Bm=r.standard_normal((B, L, N)),
        Cm=r.standard_normal((B, L, N)), A=-r.uniform(0.2, 4.0, (D, N)),
        Dskip=r.standard_normal(D), dt_bias=r.standard_normal(D) - 1.0,
        h0=r.standard_normal((B, D, N)) if with_h0 else None)
    return c


def run_scan(c, **kw):
    args = dict(x=c["x"], dt=c["dt"], A=c["A"], Bm=c["Bm"], Cm=c["Cm"], Dskip=c["Dskip"],
                z=c["z"], dt_bias=c["dt_bias"], h0=c["h0"])
    args.update(kw)
    return oracle.scan_fwd(**args)


# ---------------------------------------------------------------- P10: softplus, silu
def test_softplus_matches_logaddexp():
    # N=1, A=0, h0=0, B=C=1, D=0, x=1, no gate, L=1  =>  out = delta = softplus(dt + dt_bias)
    v = np.concatenate([np.linspace(-40, 40, 321), [-745.0, -700.0, -100.0, 100.0, 700.0, 0.0]])
    n = v.size
    one = np.ones((n, 1, 1))
    bias = np.array([0.37])
    out, hf = oracle.scan_fwd(x=one, dt=(v - 0.37).reshape(n, 1, 1), A=np.zeros((1, 1)),
                              Bm=one, Cm=one, dt_bias=bias, dt_softplus=True)
    ref = np.logaddexp(0.0, (v - 0.37) + 0.37)
    np.testing.assert_allclose(out.ravel(), ref, rtol=1e-14, atol=0)
    np.testing.assert_allclose(hf.ravel(), ref, rtol=1e-14, atol=0)
    # flag off: delta is dt + dt_bias itself
    out2, _ = oracle.scan_fwd(x=one, dt=(v - 0.37).reshape(n, 1, 1), A=np.zeros((1, 1)),
                              Bm=one, Cm=one, dt_bias=bias, dt_softplus=False)
    np.testing.assert_allclose(out2.ravel(), (v - 0.37) + 0.37, rtol=1e-15, atol=0)


def test_silu_gate_matches_expit():
    # C = 0, D = 1, x = 1  =>  out = silu(z) = z * expit(z)
    zv = np.concatenate([np.linspace(-30, 30, 241), [-700.0, 700.0]])
    n = zv.size
    one = np.ones((n, 1, 1))
    out, _ = oracle.scan_fwd(x=one, dt=one, A=-np.ones((1, 2)), Bm=np.ones((n, 1, 2)),
                             Cm=np.zeros((n, 1, 2)), Dskip=np.ones(1), z=zv.reshape(n, 1, 1))
    np.testing.assert_allclose(out.ravel(), zv * expit(zv), rtol=1e-14, atol=1e-300)


def test_inverse_softplus_round_trip_of_generator():
    # the generator's dt_bias is the inverse softplus of a log-uniform dt0 in [1e-3, 0.1]
    p = synth.layer_params(rnd(5), 512, 16, 4)
    dt0 = np.logaddexp(0.0, p["dt_bias"].astype(np.float64))
    assert dt0.min() > 1e-3 * 0.999 and dt0.max() < 0.1 * 1.001
    lg = np.log(dt0)
    assert abs(lg.mean() - 0.5 * (np.log(1e-3) + np.log(0.1))) < 0.2   # log-uniform, not uniform


# ---------------------------------------------------------------- P1: geometric series
@pytest.mark.parametrize("softplus", [False, True])
def test_constant_inputs_geometric_series(softplus):
    L, D, N = 50, 3, 5
    r = rnd(11)
    xc = r.standard_normal(D)
    bc = r.standard_normal(N)
    cc = r.standard_normal(N)
    A = -r.uniform(0.1, 3.0, (D, N))
    Dk = r.standard_normal(D)
    zc = r.standard_normal(D)
    h0 = r.standard_normal((1, D, N))
    if softplus:
        dtc = r.standard_normal(D)
        bias = r.standard_normal(D)
        delta = np.logaddexp(0.0, dtc + bias)
    else:
        dtc = r.uniform(0.01, 0.5, D)
        bias = np.zeros(D)
        delta = dtc
    tile = lambda v, n: np.broadcast_to(v, (1, L, n)).copy()
    out, hf = oracle.scan_fwd(x=tile(xc, D), dt=tile(dtc, D), A=A, Bm=tile(bc, N), Cm=tile(cc, N),
                              Dskip=Dk, z=tile(zc, D), dt_bias=bias, h0=h0, dt_softplus=softplus)
    abar = np.exp(delta[:, None] * A)                                  # (D,N)
    t1 = np.arange(1, L + 1)[:, None, None]                            # t+1
    pw = abar[None] ** t1                                              # (L,D,N)
    h = pw * h0 + (delta[:, None] * bc[None, :] * xc[:, None])[None] * (1 - pw) / (1 - abar)[None]
    y = (h * cc[None, None, :]).sum(-1) + Dk * xc
    ref = y * (zc * expit(zc))
    np.testing.assert_allclose(out[0], ref, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(hf[0], h[-1], rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- P2: A = 0 -> cumulative sum
def test_A_zero_reduces_to_cumsum():
    c = rand_case(21, B=2, L=33, D=4, N=3)
    c["A"] = np.zeros_like(c["A"])
    out, hf = run_scan(c, z=None, Dskip=None)
    delta = np.logaddexp(0.0, c["dt"] + c["dt_bias"])
    inc = (delta * c["x"])[:, :, :, None] * c["Bm"][:, :, None, :]      # (B,L,D,N)
    h = c["h0"][:, None] + np.cumsum(inc, axis=1)
    y = np.einsum("bldn,bln->bld", h, c["Cm"])
    np.testing.assert_allclose(out, y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(hf, h[:, -1], rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- P3: unrolled form, tiny
def unrolled(c, softplus=True):
    """h_t[n] = exp(A_n S_t) h0 + sum_{s<=t} exp(A_n (S_t - S_s)) delta_s B_s[n] x_s with
    S_t = sum_{r<=t} delta_r; written as explicit sums, not as a recurrence."""
    x, Bm, Cm, A = c["x"], c["Bm"], c["Cm"], c["A"]
    Bn, L, D = x.shape
    N = A.shape[1]
    v = c["dt"] + (c["dt_bias"] if c["dt_bias"] is not None else 0.0)
    delta = np.logaddexp(0.0, v) if softplus else v
    h0 = c["h0"] if c["h0"] is not None else np.zeros((Bn, D, N))
    out = np.zeros((Bn, L, D))
    hlast = np.zeros((Bn, D, N))
    for b in range(Bn):
        for d in range(D):
            S = np.cumsum(delta[b, :, d])
            for t in range(L):
                y = 0.0
                for n in range(N):
                    h = np.exp(A[d, n] * S[t]) * h0[b, d, n]
                    for s in range(t + 1):
                        h += np.exp(A[d, n] * (S[t] - S[s])) * delta[b, s, d] * Bm[b, s, n] * x[b, s, d]
                    y += Cm[b, t, n] * h
                    if t == L - 1:
                        hlast[b, d, n] = h
                if c["Dskip"] is not None:
                    y += c["Dskip"][d] * x[b, t, d]
                if c["z"] is not None:
                    y *= c["z"][b, t, d] * expit(c["z"][b, t, d])
                out[b, t, d] = y
    return out, hlast


@pytest.mark.parametrize("seed,softplus", [(1, True), (2, False), (3, True)])
def test_unrolled_brute_force(seed, softplus):
    c = rand_case(seed, B=2, L=8, D=3, N=4, with_h0=(seed != 3))
    if not softplus:
        c["dt"] = np.abs(c["dt"]) + 0.05
        c["dt_bias"] = np.abs(c["dt_bias"]) * 0.1
    out, hf = run_scan(c, dt_softplus=softplus)
    ro, rh = unrolled(c, softplus)
    np.testing.assert_allclose(out, ro, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(hf, rh, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- P4: scan == repeated step
def test_scan_equals_repeated_steps():
    c = rand_case(31, B=3, L=19, D=5, N=4)
    out, hf = run_scan(c)
    h = c["h0"].copy()
    for t in range(19):
        h, o = oracle.state_step(h, c["x"][:, t], c["dt"][:, t], c["A"], c["Bm"][:, t], c["Cm"][:, t],
                                 Dskip=c["Dskip"], z=c["z"][:, t], dt_bias=c["dt_bias"])
        np.testing.assert_allclose(o, out[:, t], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(h, hf, rtol=1e-13, atol=1e-14)


def test_step_parent_index_reads_parent_state():
    # a step with parent p must equal a step on the explicitly gathered states
    r = rnd(33)
    n_in, n_out, D, N = 4, 9, 3, 5
    h_in = r.standard_normal((n_in, D, N))
    parent = r.integers(0, n_in, n_out).astype(np.int32)
    tok = dict(x=r.standard_normal((n_out, D)), dt=r.standard_normal((n_out, D)),
               Bm=r.standard_normal((n_out, N)), Cm=r.standard_normal((n_out, N)))
    A = -r.uniform(0.1, 2, (D, N))
    h1, o1 = oracle.state_step(h_in, A=A, parent=parent, **tok)
    h2, o2 = oracle.state_step(h_in[parent], A=A, parent=None, **tok)
    assert np.array_equal(h1, h2) and np.array_equal(o1, o2)
    # and against the one-step closed form h' = exp(delta A) h_p + delta B x ; y = C.h'
    delta = np.logaddexp(0, tok["dt"])
    href = np.exp(delta[:, :, None] * A[None]) * h_in[parent] + \
        (delta * tok["x"])[:, :, None] * tok["Bm"][:, None, :]
    np.testing.assert_allclose(h1, href, rtol=1e-14)
    np.testing.assert_allclose(o1, np.einsum("jdn,jn->jd", href, tok["Cm"]), rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- P5: chunk carry
@pytest.mark.parametrize("L1", [1, 5, 12])
def test_scan_chunk_carry(L1):
    c = rand_case(41, B=2, L=13, D=4, N=3)
    out, hf = run_scan(c)
    sl = lambda k, a, b: c[k][:, a:b]
    cut = lambda a, b, h0: oracle.scan_fwd(sl("x", a, b), sl("dt", a, b), c["A"], sl("Bm", a, b),
                                           sl("Cm", a, b), c["Dskip"], sl("z", a, b), c["dt_bias"], h0)
    o1, h1 = cut(0, L1, c["h0"])
    o2, h2 = cut(L1, 13, h1)
    np.testing.assert_allclose(np.concatenate([o1, o2], 1), out, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(h2, hf, rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("K", [2, 3, 4])
@pytest.mark.parametrize("L1", [1, 2, 7])
def test_conv_chunk_carry(K, L1):
    r = rnd(43)
    B, L, D = 2, 11, 5
    x = r.standard_normal((B, L, D))
    w = r.standard_normal((D, K))
    bias = r.standard_normal(D)
    st0 = r.standard_normal((B, D, K - 1))
    y, st = oracle.conv1d_fwd(x, w, bias, st0)
    y1, s1 = oracle.conv1d_fwd(x[:, :L1], w, bias, st0)
    y2, s2 = oracle.conv1d_fwd(x[:, L1:], w, bias, s1)
    assert np.array_equal(np.concatenate([y1, y2], 1), y)
    assert np.array_equal(s2, st)


# ---------------------------------------------------------------- P6: delta -> 0
def test_delta_to_zero_leaves_state_unchanged():
    c = rand_case(51, B=2, L=9, D=4, N=3)
    c["dt"] = np.full_like(c["dt"], -1e4)
    c["dt_bias"] = np.zeros_like(c["dt_bias"])
    out, hf = run_scan(c, z=None)
    assert np.array_equal(hf, c["h0"])                       # exactly unchanged
    y = np.einsum("bdn,bln->bld", c["h0"], c["Cm"]) + c["Dskip"] * c["x"]
    np.testing.assert_allclose(out, y, rtol=1e-13, atol=1e-14)


# ---------------------------------------------------------------- P7: linearity in x
def test_linear_in_x_from_zero_state():
    c = rand_case(61, B=1, L=15, D=4, N=4, with_h0=False)
    x2 = rnd(62).standard_normal(c["x"].shape)
    a, b = 0.7, -1.9
    o1, h1 = run_scan(c)
    o2, h2 = run_scan(c, x=x2)
    o3, h3 = run_scan(c, x=a * c["x"] + b * x2)
    np.testing.assert_allclose(o3, a * o1 + b * o2, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(h3, a * h1 + b * h2, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- P8: special cases
def test_special_cases():
    c = rand_case(71, B=2, L=6, D=3, N=4)
    o, _ = run_scan(c, Cm=np.zeros_like(c["Cm"]))
    np.testing.assert_allclose(o, c["Dskip"] * c["x"] * c["z"] * expit(c["z"]), rtol=1e-13, atol=1e-15)
    o_gate, h_gate = run_scan(c)
    o_nogate, h_nogate = run_scan(c, z=None)
    np.testing.assert_allclose(o_gate, o_nogate * c["z"] * expit(c["z"]), rtol=1e-13, atol=1e-15)
    assert np.array_equal(h_gate, h_nogate)                  # the gate does not touch the state
    o_noskip, _ = run_scan(c, z=None, Dskip=None)
    np.testing.assert_allclose(o_nogate - o_noskip, c["Dskip"] * c["x"], rtol=1e-9, atol=1e-12)
    o_z0, _ = run_scan(c, z=np.zeros_like(c["z"]))
    assert np.all(o_z0 == 0)
    o_nb, _ = run_scan(c, dt_bias=None)
    o_zb, _ = run_scan(c, dt_bias=np.zeros_like(c["dt_bias"]))
    assert np.array_equal(o_nb, o_zb)
    assert not np.allclose(o_nb, o_gate)                     # dt_bias is really used
    o_h0none, _ = run_scan(c, h0=None)
    o_h0zero, _ = run_scan(c, h0=np.zeros_like(c["h0"]))
    assert np.array_equal(o_h0none, o_h0zero)
    # batches are independent and B/C are per batch row
    ob, hb = oracle.scan_fwd(c["x"][1:], c["dt"][1:], c["A"], c["Bm"][1:], c["Cm"][1:], c["Dskip"],
                             c["z"][1:], c["dt_bias"], c["h0"][1:])
    assert np.array_equal(ob, o_gate[1:]) and np.array_equal(hb, h_gate[1:])
    # empty sequence: state passes through
    e = lambda k: c[k][:, :0]
    oe, he = oracle.scan_fwd(e("x"), e("dt"), c["A"], e("Bm"), e("Cm"), c["Dskip"], e("z"),
                             c["dt_bias"], c["h0"])
    assert oe.shape == (2, 0, 3) and np.array_equal(he, c["h0"])


# ---------------------------------------------------------------- P9: conv
@pytest.mark.parametrize("K", [1, 2, 3, 4])
def test_conv_matches_numpy_convolve_and_toeplitz(K):
    r = rnd(81)
    B, L, D = 2, 17, 4
    x = r.standard_normal((B, L, D))
    w = r.standard_normal((D, K))
    bias = r.standard_normal(D)
    y, st = oracle.conv1d_fwd(x, w, bias, None, apply_silu=False)
    for b in range(B):
        for d in range(D):
            # causal correlation with taps w[d,0..K-1] on x[t-K+1..t] == convolution with reversed taps
            ref = np.convolve(x[b, :, d], w[d, ::-1])[:L] + bias[d]
            np.testing.assert_allclose(y[b, :, d], ref, rtol=1e-12, atol=1e-13)
            T = np.zeros((L, L))
            for t in range(L):
                for k in range(K):
                    s = t - (K - 1) + k
                    if s >= 0:
                        T[t, s] = w[d, k]
            np.testing.assert_allclose(y[b, :, d], T @ x[b, :, d] + bias[d], rtol=1e-12, atol=1e-13)
    ys, _ = oracle.conv1d_fwd(x, w, bias, None, apply_silu=True)
    np.testing.assert_allclose(ys, y * expit(y), rtol=1e-13, atol=1e-15)
    assert np.array_equal(st, np.transpose(x[:, L - (K - 1):, :], (0, 2, 1)).reshape(B, D, K - 1))


def test_conv_one_hot_tap_is_a_delay_and_state_is_left_context():
    r = rnd(83)
    B, L, D, K = 1, 9, 2, 4
    x = r.standard_normal((B, L, D))
    st0 = r.standard_normal((B, D, K - 1))
    for k in range(K):
        w = np.zeros((D, K))
        w[:, k] = 1.0
        y, st = oracle.conv1d_fwd(x, w, None, st0, apply_silu=False)
        xpad = np.concatenate([np.transpose(st0, (0, 2, 1)), x], axis=1)     # (B, K-1+L, D)
        assert np.array_equal(y, xpad[:, k:k + L])                            # delay by K-1-k
        assert np.array_equal(st, np.transpose(xpad[:, L:], (0, 2, 1)))
    # no bias and no state == zero bias and zero state
    w = r.standard_normal((D, K))
    ya, _ = oracle.conv1d_fwd(x, w, None, None)
    yb, _ = oracle.conv1d_fwd(x, w, np.zeros(D), np.zeros((B, D, K - 1)))
    assert np.array_equal(ya, yb)


@pytest.mark.parametrize("L", [0, 1, 2])
def test_conv_shorter_than_window(L):
    r = rnd(85)
    B, D, K = 2, 3, 4
    x = r.standard_normal((B, L, D))
    st0 = r.standard_normal((B, D, K - 1))
    w = r.standard_normal((D, K))
    y, st = oracle.conv1d_fwd(x, w, None, st0, apply_silu=False)
    xpad = np.concatenate([np.transpose(st0, (0, 2, 1)), x], axis=1)
    for t in range(L):
        np.testing.assert_allclose(y[:, t], np.einsum("bkd,dk->bd", xpad[:, t:t + K], w), rtol=1e-13)
    assert np.array_equal(st, np.transpose(xpad[:, L:L + K - 1], (0, 2, 1)))


# ---------------------------------------------------------------- P11, P12: fork
def test_fork_is_fancy_indexing_bytes():
    r = rnd(91)
    nl, n_in, n_out, D, N, K = 3, 5, 8, 6, 4, 4
    conv = r.integers(0, 2 ** 16, (nl, n_in, D, K - 1)).astype(np.uint16)     # bf16 bit patterns
    ssm = r.standard_normal((nl, n_in, D, N)).astype(np.float32)
    ssm.view(np.uint32)[0, 0, 0, 0] = 0x7FC12345                              # NaN payload survives
    parent = r.integers(0, n_in, n_out).astype(np.int32)
    cd, sd = oracle.state_fork(conv, ssm, parent)
    assert cd.tobytes() == conv[:, parent].tobytes()
    assert sd.tobytes() == ssm[:, parent].tobytes()
    ci, si = oracle.state_fork(conv, ssm, np.arange(n_in, dtype=np.int32))
    assert ci.tobytes() == conv.tobytes() and si.tobytes() == ssm.tobytes()
    cb, sb = oracle.state_fork(conv, ssm, np.full(7, 2, dtype=np.int32))
    assert all(sb[:, j].tobytes() == ssm[:, 2].tobytes() for j in range(7))
    c_only, none = oracle.state_fork(conv, None, parent)
    assert none is None and c_only.tobytes() == cd.tobytes()


def read_golden_trees():
    rows = []
    with open(os.path.join(GOLDEN, "tree_configs.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            t, b = line.split("|")
            rows.append((tuple(int(v) for v in t.split(",")), [int(v) for v in b.split(",")]))
    return rows


def test_paper_tree_shapes_and_fork_chain():
    rows = read_golden_trees()
    assert ((3, 2, 2, 1, 1), [3, 6, 12, 12, 12]) in rows
    r = rnd(93)
    D, N, K = 4, 3, 4
    for tree, sizes in rows:
        assert oracle_tree.tree_batch_sizes(tree) == sizes
        parents = oracle_tree.tree_parents(tree)
        ssm = r.standard_normal((2, 1, D, N)).astype(np.float32)          # root: one state per layer
        conv = r.standard_normal((2, 1, D, K - 1)).astype(np.float32)
        copies = 0
        prev = 1
        for n_i, b_i, par in zip(tree, sizes, parents):
            assert par.shape == (b_i,) and par.max() == prev - 1
            assert np.array_equal(np.bincount(par, minlength=prev), np.full(prev, n_i))
            conv, ssm = oracle.state_fork(conv, ssm, par)
            assert ssm.shape == (2, b_i, D, N)
            copies += b_i
            prev = b_i
        assert copies == sum(sizes)
        # nothing but copies happened: every leaf still equals the root state, siblings identical
        assert all(ssm[:, j].tobytes() == ssm[:, 0].tobytes() for j in range(prev))


def test_bf16_widening_is_exact():
    r = rnd(95)
    f = r.standard_normal(1000).astype(np.float32)
    bits = synth.f32_to_bf16_bits(f)
    back = synth.bf16_bits_to_f32(bits)
    assert np.array_equal(oracle.widen(bits, bf16=True), back.astype(np.float64))
    # round to nearest even: error at most half a bf16 ulp, and values already in bf16 survive
    assert np.all(np.abs(back - f) <= np.abs(f) * 2.0 ** -8)
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)
    tie = np.array([0x3F808000, 0x3F818000], dtype=np.uint32).view(np.float32)   # exact ties
    assert list(synth.f32_to_bf16_bits(tie)) == [0x3F80, 0x3F82]


def test_round_bf16_of_the_block_oracle():
    """oracle._round_bf16 (the rounding a stage's stored tensor gets) against what the bfloat16 format fixes: a
    bfloat16 keeps the sign, the 8 exponent bits and the top 7 fraction bits of a float32, nearest value, ties to
    the even fraction.  Truncation, rounding half up and rounding half away from zero each fail a line below."""
    rb = oracle._round_bf16
    # known values, worked by hand from their float32 bit patterns
    #   pi  = 0x40490FDB -> 0x4049 (low half below 0x8000: down)  = 3.140625
    #   0.1 = 0x3DCCCCCD -> 0x3DCD (low half above 0x8000: up)    = 0.10009765625
    #   1/3 = 0x3EAAAAAB -> 0x3EAB (up)                           = 0.333984375
    got = rb(np.array([np.pi, 0.1, 1.0 / 3.0, -0.1]))
    assert got.tolist() == [3.140625, 0.10009765625, 0.333984375, -0.10009765625]
    # exact ties between neighbours 1 + k 2^-7: to the even fraction, for either sign
    ties = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 5 * 2.0 ** -8, -(1 + 2.0 ** -8), -(1 + 3 * 2.0 ** -8)])
    assert rb(ties).tolist() == [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -6, -1.0, -(1 + 2.0 ** -6)]
    # just off a tie: to the nearer neighbour
    assert rb(np.array([1 + 2.0 ** -8 + 2.0 ** -20, 1 + 2.0 ** -8 - 2.0 ** -20])).tolist() == [1 + 2.0 ** -7, 1.0]
    # values that are bfloat16 already (8 significant bits, any exponent) are fixed points; the result always is one
    r = rnd(96)
    exact = np.ldexp(r.integers(128, 256, 500).astype(np.float64), r.integers(-60, 60, 500)) * r.choice([-1.0, 1.0], 500)
    assert np.array_equal(rb(exact), exact)
    x = r.standard_normal(4000) * np.exp(r.uniform(-20, 20, 4000))
    y = rb(x)
    assert np.array_equal(rb(y), y)
    mant, _ = np.frexp(y)
    assert np.array_equal(mant * 256, np.round(mant * 256))                  # 8 significant bits
    # nearest: within half a unit in the last place (2^-9 relative to the power of two below |x|), some on either side
    ulp = np.ldexp(1.0, np.floor(np.log2(np.abs(x))).astype(int) - 7)
    assert np.all(np.abs(y - x) <= 0.5 * ulp)
    assert (np.abs(y) > np.abs(x)).any() and (np.abs(y) < np.abs(x)).any()
    # carry out of the fraction: just below a power of two rounds up to it
    assert rb(np.array([1.99999, 255.9])).tolist() == [2.0, 256.0]
    assert rb(np.array([0.0, -0.0])).tolist() == [0.0, 0.0] and rb(np.zeros((2, 3))).shape == (2, 3)


# ---------------------------------------------------------------- dense parts of the block
def test_linear_against_explicit_sums():
    r = rnd(101)
    M, N, K = 5, 4, 7
    x, w, b, res = r.standard_normal((M, K)), r.standard_normal((N, K)), r.standard_normal(N), r.standard_normal((M, N))
    out = oracle.linear(x, w, b, res)
    for m in range(M):
        for n in range(N):
            s = sum(x[m, k] * w[n, k] for k in range(K)) + b[n] + res[m, n]
            assert out[m, n] == pytest.approx(s, rel=1e-13, abs=1e-13)
    assert np.array_equal(oracle.linear(x, np.eye(K)), x)              # identity weights
    assert oracle.linear(x, w).shape == (M, N)


def test_rmsnorm_closed_forms():
    r = rnd(103)
    C = 16
    w = r.standard_normal(C)
    # a constant row c: mean square c^2, so y = w * c / sqrt(c^2 + eps)
    y = oracle.rmsnorm(np.full((1, C), 3.0), w, 0.5)
    np.testing.assert_allclose(y[0], w * 3.0 / np.sqrt(9.5), rtol=1e-14)
    # eps = 0: scale invariant, and the normalized row has unit mean square before the weight
    x = r.standard_normal((4, C))
    np.testing.assert_allclose(oracle.rmsnorm(7.0 * x, w, 0.0), oracle.rmsnorm(x, w, 0.0), rtol=1e-13)
    np.testing.assert_allclose(np.mean(oracle.rmsnorm(x, np.ones(C), 0.0) ** 2, axis=1), 1.0, rtol=1e-13)
    # a one-hot row e_j * a: mean square a^2 / C
    e = np.zeros((1, C))
    e[0, 5] = -2.0
    y = oracle.rmsnorm(e, w, 0.0)
    assert y[0, 5] == pytest.approx(-np.sqrt(C) * w[5], rel=1e-14) and np.count_nonzero(y) == 1


def test_topk_and_embedding_reduce_to_library_routines():
    r = rnd(107)
    x = r.standard_normal((6, 50))
    x[2, 7] = x[2, 31] = x[2].max() + 1.0                  # a tie at the top: the lower index first
    x[3, 5] = np.nan
    idx, val = oracle.topk(x, 4)
    for m in range(6):
        row = np.where(np.isnan(x[m]), -np.inf, x[m])
        assert np.array_equal(val[m], np.sort(row)[::-1][:4])
        assert np.array_equal(row[idx[m]], val[m]) and len(set(idx[m])) == 4
    assert list(idx[2, :2]) == [7, 31] and 5 not in idx[3]
    i2, v2 = oracle.topk(np.array([[1.0, 3.0]]), 3)
    assert list(i2[0]) == [1, 0, -1] and v2[0, 2] == -np.inf
    table = r.standard_normal((9, 4))
    tok = np.array([3, 3, 0, 8])
    assert np.array_equal(oracle.embedding(tok, table), np.stack([table[3], table[3], table[0], table[8]]))


def _block_weights64(rng, dm, D, N, K, R):
    return dict(norm_w=rng.uniform(0.5, 1.5, dm), in_proj_w=rng.standard_normal((2 * D, dm)) / np.sqrt(dm),
                conv_w=rng.standard_normal((D, K)), conv_b=rng.standard_normal(D),
                x_proj_w=rng.standard_normal((R + 2 * N, D)) / np.sqrt(D), dt_proj_w=rng.standard_normal((D, R)),
                dt_bias=rng.standard_normal(D) - 1.0, A=-rng.uniform(0.2, 4.0, (D, N)), Dskip=rng.standard_normal(D),
                out_proj_w=rng.standard_normal((dm, D)) / np.sqrt(D))


def test_block_single_token_from_zero_state_is_an_explicit_expression():
    """Wiring of the block (Sec. 3.1, the Mamba block of the drafter): for one token and zero carried
    states nothing recurs, so every output is a plain expression of the weights.  The conv sees only its
    newest tap; the state is delta * x_c * B; the order x | z of in_proj's halves and dt | B | C of
    x_proj's rows, the low-rank dt projection and the gate all show in the result.  Evaluated in
    float64 throughout (no rounding between stages)."""
    rng = rnd(31)
    dm, D, N, K, R = 5, 6, 4, 4, 2
    w = _block_weights64(rng, dm, D, N, K, R)
    hid = rng.standard_normal((3, 1, dm))
    out, conv_state, h = oracle.block_fwd(w, hid, round_between=False)
    v = hid[:, 0]
    u = v / np.sqrt(np.mean(v * v, axis=1, keepdims=True) + 1e-5) * w["norm_w"]
    x, z = u @ w["in_proj_w"][:D].T, u @ w["in_proj_w"][D:].T
    pre = x * w["conv_w"][:, K - 1] + w["conv_b"]
    xc = pre * expit(pre)
    low, Bv, Cv = xc @ w["x_proj_w"][:R].T, xc @ w["x_proj_w"][R:R + N].T, xc @ w["x_proj_w"][R + N:].T
    delta = np.logaddexp(0.0, low @ w["dt_proj_w"].T + w["dt_bias"])
    h_want = (delta * xc)[:, :, None] * Bv[:, None, :]
    y = (np.einsum("bdn,bn->bd", h_want, Cv) + w["Dskip"] * xc) * (z * expit(z))
    np.testing.assert_allclose(h, h_want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out[:, 0], v + y @ w["out_proj_w"].T, rtol=1e-12, atol=1e-13)
    # the carried conv inputs: the x half before the conv, newest last, zeros in front of the sequence
    assert conv_state.shape == (3, D, K - 1)
    np.testing.assert_allclose(conv_state[:, :, K - 2], x, rtol=1e-12, atol=1e-13)
    assert not conv_state[:, :, :K - 2].any()


def test_block_degenerate_weights_and_causality():
    """(a) out_proj = 0 leaves the residual stream unchanged; (b) so does a zero z half of in_proj (the gate
    silu(0) is 0), while a zero x half with zero conv bias does too but a zero x half with a conv bias does
    not (the two halves are not interchangeable); (c) a token changes no output before it, and the states a
    split run carries make the second half equal the one-pass result; (d) rounding between the stages moves
    the result a little (six roundings of 2^-9 each, amplified by the weights) and not by nothing."""
    rng = rnd(32)
    dm, D, N, K, R = 8, 12, 4, 3, 2
    w = _block_weights64(rng, dm, D, N, K, R)
    hid = rng.standard_normal((2, 9, dm))
    full, cs, hs = oracle.block_fwd(w, hid, round_between=False)
    assert np.max(np.abs(full - hid)) > 1e-2
    assert np.array_equal(oracle.block_fwd(dict(w, out_proj_w=0 * w["out_proj_w"]), hid, round_between=False)[0], hid)
    wz = dict(w, in_proj_w=np.concatenate([w["in_proj_w"][:D], np.zeros((D, dm))]))
    assert np.array_equal(oracle.block_fwd(wz, hid, round_between=False)[0], hid)
    wx = dict(w, in_proj_w=np.concatenate([np.zeros((D, dm)), w["in_proj_w"][D:]]))
    assert np.max(np.abs(oracle.block_fwd(wx, hid, round_between=False)[0] - hid)) > 1e-3
    assert np.array_equal(oracle.block_fwd(dict(wx, conv_b=np.zeros(D)), hid, round_between=False)[0], hid)
    hid2 = hid.copy()
    hid2[:, 5] += 1.0
    other = oracle.block_fwd(w, hid2, round_between=False)[0]
    assert np.array_equal(other[:, :5], full[:, :5]) and np.min(np.max(np.abs(other[:, 5:] - full[:, 5:]), axis=2)) > 0
    o1, c1, s1 = oracle.block_fwd(w, hid[:, :4], round_between=False)
    o2, c2, s2 = oracle.block_fwd(w, hid[:, 4:], conv_state_in=c1, h0=s1, round_between=False)
    np.testing.assert_allclose(np.concatenate([o1, o2], axis=1), full, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(c2, cs, rtol=0, atol=0)
    np.testing.assert_allclose(s2, hs, rtol=1e-12, atol=1e-13)
    rounded = oracle.block_fwd(w, hid, round_between=True)[0]
    assert 0 < np.max(np.abs(rounded - full)) <= 0.1 * np.sqrt(np.mean(full ** 2))


def test_drafter_tree_reduces_to_greedy_decoding_and_to_prefill():
    """The drafter oracle against what it must reduce to: (a) along a (1, 1, 1) tree it is greedy
    decoding, so encoding prefix + drafted tokens in one pass gives the same next-token logits
    (the recurrent step and the sequence form agree, Sec. 3.1); (b) the first child of every node of
    a wider tree is the greedy path; (c) children of one parent start from the same states, so two
    siblings that are fed the same token would agree: checked through the parents' j // N_i order by
    comparing the branch that follows the second-best first token with a fresh run on that token."""
    from oracle import drafter as od
    from paper_2506_01206_amd import synth
    rng = np.random.default_rng(5)
    V, dm, D, N, K, R, nl = 40, 32, 64, 8, 4, 4, 2
    wid = lambda a: oracle.widen(a, bf16=(a.dtype == np.uint16))
    w = dict(embedding=wid(synth.f32_to_bf16_bits(rng.standard_normal((V, dm)).astype(np.float32))),
             lm_head=wid(synth.f32_to_bf16_bits(rng.standard_normal((V, dm)).astype(np.float32))),
             norm_f=np.ones(dm), blocks=[{k: wid(v) for k, v in synth.block_weights(rng, dm, D, N, K, R).items()}
                                         for _ in range(nl)])
    prefix = rng.integers(0, V, 12).astype(np.int32)
    lg, cs, hs = od.prefill(w, prefix)
    tok, logits, _ = od.draft(w, (1, 1, 1), lg, cs, hs)
    assert tok[0][0] == np.argmax(lg[0])
    greedy = np.concatenate([prefix] + tok)
    for i in range(3):
        again, _, _ = od.prefill(w, greedy[:len(prefix) + i + 1])
        rms = np.sqrt(np.mean(again ** 2))
        assert np.max(np.abs(again - logits[i])) <= 2e-2 * rms          # a bf16 rounding flip at most
    wide, wl, _ = od.draft(w, (2, 2, 1), lg, cs, hs)
    assert [int(t[0]) for t in wide] == [int(t[0]) for t in tok]          # branch 0 is the greedy path
    assert [t.size for t in wide] == [2, 4, 4]
    # branch 1 at depth 1 carries the second-best first token; rows 2, 3 at depth 2 are its children
    second = int(wide[0][1])
    lg2, _, _ = od.prefill(w, np.concatenate([prefix, [second]]).astype(np.int32))
    order = np.argsort(-lg2[0], kind="stable")[:2]
    assert list(wide[1][2:4]) == list(order)


# ------------------------------------------------------------------------------------ Mamba-2 style core
def _ssd_case(rng, B, L, H, P, N):
    return dict(x=rng.standard_normal((B, L, H, P)), z=rng.standard_normal((B, L, H, P)),
                dt=0.5 * rng.standard_normal((B, L, H)), Bm=rng.standard_normal((B, L, N)), Cm=rng.standard_normal((B, L, N)),
                A=-rng.uniform(0.3, 4.0, H), Dskip=rng.standard_normal(H), dt_bias=rng.uniform(-3, 0, H),
                h0=rng.standard_normal((B, H, P, N)))


def test_ssd_oracle_is_the_selective_scan_with_one_decay_per_head():
    """The scalar-decay layer is the selective scan of the paper's drafter with A[d, n] = A[head(d)] and
    dt, D, dt_bias repeated over a head's channels: checked against the (separately pinned) C oracle."""
    from oracle import ssd
    rng = np.random.default_rng(21)
    B, L, H, P, N = 2, 37, 3, 4, 8
    c = _ssd_case(rng, B, L, H, P, N)
    out, hf = ssd.ssd_scan(c["x"], c["dt"], c["A"], c["Bm"], c["Cm"], c["Dskip"], c["z"], c["dt_bias"], c["h0"])
    rep = lambda a: np.repeat(a, P, axis=-1)
    o1, h1 = oracle.scan_fwd(c["x"].reshape(B, L, H * P), rep(c["dt"]), np.repeat(c["A"], P)[:, None] * np.ones((1, N)),
                             c["Bm"], c["Cm"], rep(c["Dskip"]), c["z"].reshape(B, L, H * P), rep(c["dt_bias"]),
                             c["h0"].reshape(B, H * P, N))
    np.testing.assert_allclose(out.reshape(B, L, H * P), o1, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(hf.reshape(B, H * P, N), h1, rtol=1e-12, atol=1e-12)


def test_ssd_oracle_against_the_dual_matrix_form_and_closed_form():
    """(a) The dual form: y_t = sum_{s<=t} (C_t . B_s) exp(sum_{r=s+1..t} delta_r A) delta_s x_s + decayed h0 term,
    written out with explicit loops on a tiny case.  (b) Constant inputs: a geometric series.
    (c) A scan equals repeated single steps, also through a parent index."""
    from oracle import ssd
    rng = np.random.default_rng(22)
    B, L, H, P, N = 1, 6, 2, 3, 4
    c = _ssd_case(rng, B, L, H, P, N)
    out, hf = ssd.ssd_scan(c["x"], c["dt"], c["A"], c["Bm"], c["Cm"], c["Dskip"], None, c["dt_bias"], c["h0"])
    delta = np.logaddexp(0.0, c["dt"] + c["dt_bias"])
    for h in range(H):
        for t in range(L):
            for p in range(P):
                y = c["Dskip"][h] * c["x"][0, t, h, p]
                for s in range(t + 1):
                    decay = np.exp(c["A"][h] * delta[0, s + 1:t + 1, h].sum())
                    y += (c["Cm"][0, t] @ c["Bm"][0, s]) * decay * delta[0, s, h] * c["x"][0, s, h, p]
                y += np.exp(c["A"][h] * delta[0, :t + 1, h].sum()) * (c["h0"][0, h, p] @ c["Cm"][0, t])
                assert abs(out[0, t, h, p] - y) < 1e-11 * max(1.0, abs(y))
    # constant inputs
    L2, d0, xv = 50, 0.3, 1.7
    bvec, cvec = rng.standard_normal(N), rng.standard_normal(N)
    x = np.full((1, L2, 1, 1), xv)
    o, hfin = ssd.ssd_scan(x, np.full((1, L2, 1), d0), np.array([-0.9]), np.tile(bvec, (1, L2, 1)), np.tile(cvec, (1, L2, 1)),
                           dt_softplus=False)
    abar = np.exp(-0.9 * d0)
    for t in (0, 7, L2 - 1):
        hn = d0 * xv * bvec * (1 - abar ** (t + 1)) / (1 - abar)
        assert abs(o[0, t, 0, 0] - cvec @ hn) < 1e-12 * max(1.0, abs(cvec @ hn))
    np.testing.assert_allclose(hfin[0, 0, 0], d0 * xv * bvec * (1 - abar ** L2) / (1 - abar), rtol=1e-12)
    # steps
    h = c["h0"]
    for t in range(L):
        h, o_t = ssd.ssd_step(h, c["x"][:, t], c["dt"][:, t], c["A"], c["Bm"][:, t], c["Cm"][:, t], c["Dskip"], None, c["dt_bias"])
        np.testing.assert_allclose(o_t, out[:, t], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(h, hf, rtol=1e-12, atol=1e-12)
    two = np.concatenate([c["h0"], 2 * c["h0"]])
    h2, _ = ssd.ssd_step(two, np.repeat(c["x"][:, 0], 3, 0), np.repeat(c["dt"][:, 0], 3, 0), c["A"], np.repeat(c["Bm"][:, 0], 3, 0),
                         np.repeat(c["Cm"][:, 0], 3, 0), parent=np.array([1, 0, 1]))
    assert np.array_equal(h2[0], h2[2]) and not np.array_equal(h2[0], h2[1])
