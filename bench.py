#!/usr/bin/env python3
"""Benchmark of the selective-SSM layer core on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
  prefill  conv1d + selective scan over the long context (Mamba-130M-shaped layer, batch 1,
           L = 32768 tokens, bf16 I/O, fp32 state), then
  decode   tree drafting over 24 such layers: 5 draft steps of 32 live branches; per draft step
           and layer one launch that forks the conv and SSM state by parent index, does the conv
           step and the state update (checked bit for bit against the three-stage path: conv-state
           fork, conv step, state step; --staged-decode times that one, 245 launches).  The 120
           launches are captured once in a HIP graph (every call has a fixed shape, which is what
           makes the paper's per-batch-size graph cache possible, Sec. 4.1) and replayed;
           --eager-decode launches them one by one.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

The roofline object covers the dominant call, the selective scan (all kernels of one call
together), timed with HIP events on the launch stream inside the timed region.  Its headline
figure is the one the task asks for: algorithmic HBM bytes per second against the 8 TB/s peak.
What actually binds the scan is the vector ALUs (one hardware exp2 and four VALU operations per
state update, and two walks over the tokens because a batch-1 sequence this long must be cut in
time), so `roofline.alu` reports fp32 operations per second against the fp32 vector peak beside
it.  `roofline.traffic` (measured HBM bytes per launch) is read from the counter summary under
profiles/.  The oracle (fp64, CPU) is timed on the same prefill for cpu_baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector, published: 256 CUs x 128 FMA lanes x 2 x 2.4 GHz

FP32_VECTOR_PLAIN_TFLOPS = 78.6   # the same without packed fp32 (this build compiles it out): 64 FMA lanes per CU and clock

# HBM bytes per scan launch from rocprofv3 counters (FETCH_SIZE + WRITE_SIZE summed over the kernels of one
# scan call, each scaled by what the same counter reads for the 1 GiB copy below): the table in this file is
# written from the counter runs whose commands it lists; a workload that has no row there reports null.
SCAN_TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "scan_hbm_traffic.md")


def scan_traffic_bytes(name):
    """Measured HBM bytes of one scan launch on synthetic config `name`, or None."""
    try:
        for line in open(SCAN_TRAFFIC_TABLE):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 4 and cells[0] == name:
                return int(round(float(cells[3]) * 1e6))
    except (OSError, ValueError):
        pass
    return None


def scan_bytes(B, L, D, N, e):
    """Algorithmic HBM bytes of one scan: x, dt, z, out (B,L,D) and Bm, Cm (B,L,N), e bytes each,
    plus A, Dskip, dt_bias once and the final state once."""
    return B * L * (4 * D + 2 * N) * e + D * N * 4 + 2 * D * 4 + B * D * N * 4


def conv_bytes(B, L, D, K, e):
    return B * L * 2 * D * e + D * K * 4 + D * 4 + B * D * (K - 1) * e


def step_bytes(nb, D, N, e):
    """One state step for nb branches: state read + write (fp32), x, dt, z, out, B, C."""
    return nb * (2 * D * N * 4 + (4 * D + 2 * N) * e) + D * N * 4 + 2 * D * 4


def scan_flops(B, L, D, N):
    """fp32 operations of the scan as it is defined (one walk over the tokens): per state update
    delta*A, exp, (delta x)*B, fma, fma = 7 (an fma counts 2, exp counts 1); per (token, channel)
    softplus 6 (add, mul, exp, add, log, mul), delta*x 1, skip fma 2, silu 5, gate 1 = 15."""
    return B * L * D * (7 * N + 15)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-wide-step", action="store_true",
                    help="skip the separate timing of the 64-branch, D=4096 state step")
    ap.add_argument("--no-block", action="store_true", help="skip the whole-block prefill timing")
    ap.add_argument("--no-scan-shapes", action="store_true",
                    help="skip the scan-only timing on the cfg1 and cfg4 prefill shapes")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time conv1d, scan, fork and step on every synthetic config (cfg0..cfg4), warm and "
                         "cold, and (unless --no-cpu-baseline) the oracle on each; adds a few minutes")
    ap.add_argument("--no-mamba2", action="store_true", help="skip the scalar-decay (Mamba-2 style) core timing")
    ap.add_argument("--no-drafter", action="store_true",
                    help="skip the whole-drafter timing (Mamba-130M shapes, prefix encoding and draft rounds)")
    ap.add_argument("--no-tree-draft", action="store_true",
                    help="skip the sequential-versus-tree draft round timing")
    ap.add_argument("--staged-decode", action="store_true",
                    help="decode leg as fork + conv step + state step (245 launches) instead of one launch per layer and step")
    ap.add_argument("--eager-decode", action="store_true",
                    help="launch the decode kernels one by one instead of replaying a HIP graph")
    ap.add_argument("--prefill", default="cfg3", help="synthetic config of the prefill leg")
    ap.add_argument("--decode", default="cfg2", help="synthetic config of the decode leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); --gpus %d is not "
              "supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_01206_amd import binding as m, synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    def to_dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    # ---------------------------------------------------------------- inputs (resident in HBM)
    pc = synth.CONFIGS[args.prefill]
    B, L, D, N, K = pc["batch"], pc["L"], pc["D"], pc["N"], pc["K"]
    e = 2 if pc["io"] == synth.BF16 else 4
    case = synth.config_prefill(args.prefill)
    P = {k: to_dev(case[k]) for k in ("x", "z", "Bm", "Cm", "dt", "A", "Dskip", "dt_bias", "conv_w",
                                       "conv_bias")}
    xc = torch.empty_like(P["x"])
    conv_state = torch.empty((B, D, K - 1), dtype=P["x"].dtype, device=dev)
    out = torch.empty_like(P["x"])
    h_final = torch.empty((B, D, N), dtype=torch.float32, device=dev)
    ws_bytes = m.mamba_scan_workspace_bytes(B, L, D, N, 0)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    dcfg = synth.CONFIGS[args.decode]
    nl = dcfg.get("n_layers", 24)
    dc = synth.decode_case(nl, dcfg["branches"], dcfg["steps"], dcfg["D"], dcfg["N"], dcfg["K"],
                           dcfg["io"], synth.SEEDS[args.decode] + 100)
    nb, nsteps, Dd, Nd, Kd = dc["branches"], dc["steps"], dc["D"], dc["N"], dc["K"]
    ed = 2 if dc["io"] == synth.BF16 else 4
    LP = [{k: to_dev(v) for k, v in p.items()} for p in dc["params"]]
    TOK = [[{k: to_dev(v) for k, v in t.items()} for t in layer] for layer in dc["tokens"]]
    PAR = [to_dev(p) for p in dc["parents"]]
    # state caches: the initial states are only read; the draft steps ping-pong between two more
    ssm0, conv0 = to_dev(dc["ssm0"]), to_dev(dc["conv0"])
    ssm = [torch.empty_like(ssm0), torch.empty_like(ssm0)]
    conv = [torch.empty_like(conv0), torch.empty_like(conv0)]
    dxc = torch.empty((nb, 1, Dd), dtype=conv0.dtype, device=dev)
    dout = torch.empty((nsteps, nl, nb, Dd), dtype=conv0.dtype, device=dev)

    def prefill():
        m.mamba_conv1d_fwd(P["x"], P["conv_w"], P["conv_bias"], None, y=xc, conv_state_out=conv_state)
        m.mamba_scan_fwd(xc, P["dt"], P["A"], P["Bm"], P["Cm"], P["Dskip"], P["z"], P["dt_bias"],
                         out=out, h_final=h_final, workspace=ws)

    def decode_staged():
        # three stages: conv-state fork for all layers, then per layer a conv step and a state step (SSM fork fused in)
        src_ssm, src_conv = ssm0, conv0
        for s in range(nsteps):
            dst_ssm, dst_conv = ssm[s & 1], conv[s & 1]
            m.mamba_state_fork(src_conv, None, PAR[s], conv_dst=dst_conv)
            for l in range(nl):
                t = TOK[s][l]
                m.mamba_conv1d_fwd(t["x"].unsqueeze(1), LP[l]["conv_w"], LP[l]["conv_bias"],
                                   conv_state_in=dst_conv[l], y=dxc, conv_state_out=dst_conv[l])
                m.mamba_state_step(src_ssm[l], dxc.squeeze(1), t["dt"], LP[l]["A"], t["Bm"], t["Cm"],
                                   LP[l]["Dskip"], t["z"], LP[l]["dt_bias"], parent_idx=PAR[s],
                                   h_out=dst_ssm[l], out=dout[s, l])
            src_ssm, src_conv = dst_ssm, dst_conv

    def decode_fused():
        # one launch per layer and draft step: fork of both states, conv step and state update together
        src_ssm, src_conv = ssm0, conv0
        for s in range(nsteps):
            dst_ssm, dst_conv = ssm[s & 1], conv[s & 1]
            for l in range(nl):
                t = TOK[s][l]
                m.mamba_conv_state_step(src_ssm[l], src_conv[l], t["x"], LP[l]["conv_w"], LP[l]["conv_bias"], t["dt"],
                                        LP[l]["A"], t["Bm"], t["Cm"], LP[l]["Dskip"], t["z"], LP[l]["dt_bias"],
                                        parent_idx=PAR[s], h_out=dst_ssm[l], conv_state_out=dst_conv[l], out=dout[s, l])
            src_ssm, src_conv = dst_ssm, dst_conv

    decode_eager = decode_staged if args.staged_decode else decode_fused
    if not args.staged_decode:
        # the single launch must give what the three stages give, bit for bit
        decode_staged()
        torch.cuda.synchronize()
        st_out, st_ssm, st_conv = dout.clone(), ssm[(nsteps - 1) & 1].clone(), conv[(nsteps - 1) & 1].clone()
        dout.zero_()
        decode_fused()
        torch.cuda.synchronize()
        assert torch.equal(dout, st_out) and torch.equal(ssm[(nsteps - 1) & 1], st_ssm) and \
            torch.equal(conv[(nsteps - 1) & 1], st_conv), "fused layer step differs from fork + conv step + state step"

    ev = lambda: torch.cuda.Event(enable_timing=True)
    prefill()
    decode_eager()
    torch.cuda.synchronize()
    decode = decode_eager
    if not args.eager_decode:
        ref_out, ref_ssm = dout.clone(), ssm[(nsteps - 1) & 1].clone()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                decode_eager()
        torch.cuda.current_stream().wait_stream(side)
        decode = graph.replay
        # the replay must reproduce the eager result bit for bit, also after other work ran
        for _ in range(2):
            dout.zero_()
            prefill()
            decode()
            torch.cuda.synchronize()
            assert torch.equal(dout, ref_out) and torch.equal(ssm[(nsteps - 1) & 1], ref_ssm), \
                "HIP graph replay of the decode loop differs from the eager launches"
    for _ in range(args.warmup):
        prefill()
        decode()
    torch.cuda.synchronize()

    # ---------------------------------------------------------------- timed region
    scan_ev, conv_ev, dec_ev = [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        a, b_, c_, d_ = ev(), ev(), ev(), ev()
        a.record()
        m.mamba_conv1d_fwd(P["x"], P["conv_w"], P["conv_bias"], None, y=xc, conv_state_out=conv_state)
        b_.record()
        m.mamba_scan_fwd(xc, P["dt"], P["A"], P["Bm"], P["Cm"], P["Dskip"], P["z"], P["dt_bias"],
                         out=out, h_final=h_final, workspace=ws)
        c_.record()
        decode()
        d_.record()
        conv_ev.append((a, b_))
        scan_ev.append((b_, c_))
        dec_ev.append((c_, d_))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    scan_ms = sum(a.elapsed_time(b) for a, b in scan_ev) / args.steps
    conv_ms = sum(a.elapsed_time(b) for a, b in conv_ev) / args.steps
    dec_ms = sum(a.elapsed_time(b) for a, b in dec_ev) / args.steps

    # plain device copy of 1 GiB (read 1 GiB + write 1 GiB): the practical streaming ceiling of this
    # box, and the known-size reference the FETCH_SIZE / WRITE_SIZE counters are scaled by
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    c0, c1 = ev(), ev()
    c0.record()
    for _ in range(3):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 3 * 2 * src.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst

    # the wide decode step on its own: 64 branches of a Mamba-1.4B-shaped layer (D = 4096), parent
    # gather fused in, over rotating state buffers (> 512 MB in all) so that every launch streams
    # its state from HBM; a HIP graph of R launches is replayed to take the host out of the timing
    wide = {}
    if not args.no_wide_step:
        wc = synth.CONFIGS["cfg4"]
        wnb, wD, wN = wc["branches"], wc["D"], wc["N"]
        rngw = np.random.default_rng(404)
        wp = synth.layer_params(rngw, wD, wN, wc["K"])
        wt = {k: to_dev(v) for k, v in synth.token_inputs(rngw, (wnb,), wD, wN, wc["io"]).items()}
        wP = {k: to_dev(v) for k, v in wp.items()}
        wpar = to_dev(rngw.integers(0, wnb, wnb).astype(np.int32))
        R = int(600e6 // (wnb * wD * wN * 4)) + 1
        hin = [torch.randn((wnb, wD, wN), device=dev) for _ in range(R)]
        hout = [torch.empty((wnb, wD, wN), device=dev) for _ in range(R)]
        wout = torch.empty((wnb, wD), dtype=wt["x"].dtype, device=dev)

        def wide_round():
            for i in range(R):
                m.mamba_state_step(hin[i], wt["x"], wt["dt"], wP["A"], wt["Bm"], wt["Cm"], wP["Dskip"],
                                   wt["z"], wP["dt_bias"], parent_idx=wpar, h_out=hout[i], out=wout)
        wide_round()
        torch.cuda.synchronize()
        wg = torch.cuda.CUDAGraph()
        side2 = torch.cuda.Stream()
        side2.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side2):
            with torch.cuda.graph(wg, stream=side2):
                wide_round()
        torch.cuda.current_stream().wait_stream(side2)
        wg.replay()
        w0, w1 = ev(), ev()
        w0.record()
        for _ in range(3):
            wg.replay()
        w1.record()
        torch.cuda.synchronize()
        us = w0.elapsed_time(w1) * 1e3 / (3 * R)
        # the same rows through the library's own gather copy (mamba_state_fork): what moving the state alone costs
        def fork_round():
            for i in range(R):
                m.mamba_state_fork(None, hin[i].unsqueeze(0), wpar, ssm_dst=hout[i].unsqueeze(0))
        fork_round()
        torch.cuda.synchronize()
        fg = torch.cuda.CUDAGraph()
        side2b = torch.cuda.Stream()
        side2b.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side2b):
            with torch.cuda.graph(fg, stream=side2b):
                fork_round()
        torch.cuda.current_stream().wait_stream(side2b)
        fg.replay()
        f0, f1 = ev(), ev()
        f0.record()
        for _ in range(3):
            fg.replay()
        f1.record()
        torch.cuda.synchronize()
        fork_us = f0.elapsed_time(f1) * 1e3 / (3 * R)
        wb = step_bytes(wnb, wD, wN, 2 if wc["io"] == synth.BF16 else 4)
        wide = {"workload": "cfg4 state step: %d branches, D=%d, N=%d, %s I/O, parent gather fused, cold "
                            "(%d rotating state buffers)" % (wnb, wD, wN, wc["io"], R),
                "us_per_launch": round(us, 3), "algorithmic_bytes_per_launch": wb,
                "GBps": round(wb / us / 1e3, 1), "frac_of_hbm_peak": round(wb / us / 1e3 / HBM_PEAK_GBS, 4),
                "frac_of_copy_kernel": round(wb / us / 1e3 / copy_gbs, 4),
                "state_gather_copy_us": round(fork_us, 3),
                "state_gather_copy_note": "mamba_state_fork of the same %d state rows (%.1f MB read + written), same rotation: "
                                          "the step does the copy plus the update in %.2fx its time"
                                          % (wnb, 2 * wnb * wD * wN * 4 / 1e6, us / fork_us),
                "branch_steps_per_s_per_layer": round(wnb / (us * 1e-6), 1)}
        del hin, hout

    # the scan alone on the other prefill shapes (inputs drawn on the device with the distributions of the synthetic
    # configs): the paper's own context length on the 130M layer (cfg1), which the library scans with time across
    # lanes, and the wide batched layer (cfg4), which it scans in one pass with channels across lanes
    other_scans = {}
    if not args.no_scan_shapes:
        gs = torch.Generator(device=dev)
        gs.manual_seed(11)
        for name in ("cfg1", "cfg4"):
            c = synth.CONFIGS[name]
            cB, cL, cD, cN = c["batch"], c["L"], c["D"], c["N"]
            rnd = lambda *shape: torch.randn(*shape, device=dev, generator=gs)
            sx, sz = rnd(cB, cL, cD).to(torch.bfloat16), rnd(cB, cL, cD).to(torch.bfloat16)
            sdt = (0.1 * rnd(cB, cL, cD)).to(torch.bfloat16)
            sB, sC = rnd(cB, cL, cN).to(torch.bfloat16), rnd(cB, cL, cN).to(torch.bfloat16)
            sA = -torch.arange(1, cN + 1, device=dev, dtype=torch.float32).repeat(cD, 1).contiguous()
            dt0 = torch.exp(torch.rand(cD, device=dev, generator=gs) * (np.log(0.1) - np.log(1e-3)) + np.log(1e-3))
            sbias, sDk = dt0 + torch.log(-torch.expm1(-dt0)), torch.ones(cD, device=dev)
            so, sh = torch.empty_like(sx), torch.empty((cB, cD, cN), device=dev)
            sws = torch.empty(max(m.mamba_scan_workspace_bytes(cB, cL, cD, cN), 16), dtype=torch.uint8, device=dev)
            run_s = lambda: m.mamba_scan_fwd(sx, sdt, sA, sB, sC, sDk, sz, sbias, out=so, h_final=sh, workspace=sws)
            reps = 20 if name == "cfg1" else 5
            for _ in range(3):
                run_s()
            torch.cuda.synchronize()
            g_s = torch.cuda.CUDAGraph()
            side_s = torch.cuda.Stream()
            side_s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side_s):
                with torch.cuda.graph(g_s, stream=side_s):
                    for _ in range(reps):
                        run_s()
            torch.cuda.current_stream().wait_stream(side_s)
            g_s.replay()
            q0, q1 = ev(), ev()
            q0.record()
            for _ in range(3):
                g_s.replay()
            q1.record()
            torch.cuda.synchronize()
            s_ms = q0.elapsed_time(q1) / (3 * reps)
            nbytes = scan_bytes(cB, cL, cD, cN, 2)
            other_scans[name] = {"shape": "batch %d x L %d x D %d, N %d, bf16 I/O" % (cB, cL, cD, cN),
                                 "kernel": m.mamba_scan_kernel(cB, cL, cD, cN), "ms": round(s_ms, 5),
                                 "tokens_per_s": round(cB * cL / (s_ms * 1e-3), 1),
                                 "GBps": round(nbytes / (s_ms * 1e-3) / 1e9, 1),
                                 "frac_of_hbm_peak": round(nbytes / (s_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                 "traffic": scan_traffic_bytes(name), "algorithmic_bytes_per_launch": nbytes,
                                 "timing": "per launch in a replayed HIP graph of %d launches" % reps}
            del sx, sz, sdt, sB, sC, so, sws, g_s

    # sequential drafting (1,1,1,1,1) against the paper's default tree (3,2,2,1,1) on per-batch-size
    # state caches with one captured graph per draft position (Sec. 4.1): time of one draft round of
    # the layer core over all layers.  The paper's table on tree drafting reports the whole drafter's
    # latency growing from 6.62 to 8.30 for the same pair of shapes (other hardware, context only).
    tree_detail = {}
    if not args.no_tree_draft:
        from paper_2506_01206_amd.tree import TreeDraftCache
        for name, tree in (("sequential_1_1_1_1_1", (1, 1, 1, 1, 1)), ("tree_3_2_2_1_1", (3, 2, 2, 1, 1))):
            tc = TreeDraftCache(tree, nl, Dd, Nd, Kd, conv0.dtype, dev)
            g = torch.Generator(device=dev)
            g.manual_seed(7)
            for i in range(1, tc.gamma + 1):
                for k, buf in tc.inputs[i].items():
                    buf.copy_((torch.randn(buf.shape, device=dev, generator=g) * (0.1 if k == "dt" else 1.0)).to(buf.dtype))
            tc.set_root(conv0[:, :1], ssm0[:, :1])
            tc.draft(LP, use_graphs=False)            # loads the kernels before any capture
            tc.set_root(conv0[:, :1], ssm0[:, :1])
            tc.draft(LP, use_graphs=True)
            torch.cuda.synchronize()
            t0_, t1_ = ev(), ev()
            reps = 10
            t0_.record()
            for _ in range(reps):
                tc.draft(LP, use_graphs=True)
            t1_.record()
            torch.cuda.synchronize()
            tree_detail[name + "_ms"] = round(t0_.elapsed_time(t1_) / reps, 4)
            tree_detail[name + "_branch_steps"] = sum(tc.batch[1:]) * nl
            del tc
        tree_detail["tree_over_sequential"] = round(tree_detail["tree_3_2_2_1_1_ms"] /
                                                    tree_detail["sequential_1_1_1_1_1_ms"], 3)

    # the whole Mamba-130M-shaped block around the core (RMSNorm, in_proj, conv1d, x_proj, dt_proj, scan,
    # out_proj, residual; d_model 768, dt_rank 48) on the same prefill shape, and one decode step of it
    block_detail = {}
    if not args.no_block and pc["io"] == synth.BF16 and "dt_rank" in pc:
        dm = D // 2
        rngb = np.random.default_rng(909)
        bw = {k: to_dev(v) for k, v in synth.block_weights(rngb, dm, D, N, K, pc["dt_rank"]).items()}
        blk = m.Block(bw)
        hid = torch.randn((B, L, dm), device=dev).to(torch.bfloat16)
        hout = torch.empty_like(hid)
        bws = torch.empty(max(m.mamba_block_workspace_bytes(blk, B, L), 16), dtype=torch.uint8, device=dev)
        cso = torch.empty((B, D, K - 1), dtype=torch.bfloat16, device=dev)
        hfo = torch.empty((B, D, N), dtype=torch.float32, device=dev)
        run_blk = lambda: m.mamba_block_fwd(blk, hid, hidden_out=hout, conv_state_out=cso, h_final=hfo, workspace=bws)
        for _ in range(2):
            run_blk()
        b0, b1 = ev(), ev()
        b0.record()
        for _ in range(5):
            run_blk()
        b1.record()
        torch.cuda.synchronize()
        blk_ms = b0.elapsed_time(b1) / 5
        gemm_flops = 2.0 * B * L * (2 * D * dm + (pc["dt_rank"] + 2 * N) * D + D * pc["dt_rank"] + dm * D)
        block_detail = {"workload": "one block, %d x %d tokens, d_model %d, d_inner %d, dt_rank %d" % (B, L, dm, D, pc["dt_rank"]),
                        "prefill_ms": round(blk_ms, 4), "tokens_per_s": round(B * L / (blk_ms * 1e-3), 1),
                        "ssm_core_share": round((conv_ms + scan_ms) / blk_ms, 3),
                        "projection_GFLOP": round(gemm_flops / 1e9, 2)}
        del hid, hout, bws

    # the whole drafter at Mamba-130M shapes (Sec. 3.1: 24 blocks, d_model 768, vocabulary 50280, tied LM
    # head): encoding a 2048-token prefix, then whole draft rounds (top-N_i -> embedding -> 24 blocks
    # -> norm -> LM head per position), each round one captured HIP graph; the paper's comparison of
    # sequential against tree drafting, here with every stage of the drafter included
    drafter_detail = {}
    if not args.no_drafter:
        from paper_2506_01206_amd.drafter import MambaDrafter
        gen = torch.Generator(device=dev)
        gen.manual_seed(130)
        d_dm, d_D, d_N, d_K, d_R, d_nl, d_V, d_L = 768, 1536, 16, 4, 48, 24, 50280, 2048
        rn = lambda *shape: torch.randn(*shape, device=dev, generator=gen)
        blocks_d = []
        for _ in range(d_nl):
            dt0 = torch.exp(torch.rand(d_D, device=dev, generator=gen) * (np.log(0.1) - np.log(1e-3)) + np.log(1e-3))
            blocks_d.append(m.Block(dict(
                norm_w=1 + 0.1 * rn(d_dm), in_proj_w=(rn(2 * d_D, d_dm) / d_dm ** 0.5).to(torch.bfloat16),
                conv_w=torch.rand(d_D, d_K, device=dev, generator=gen) - 0.5, conv_b=0.1 * rn(d_D),
                x_proj_w=(rn(d_R + 2 * d_N, d_D) / d_D ** 0.5).to(torch.bfloat16),
                dt_proj_w=(rn(d_D, d_R) / d_R ** 0.5).to(torch.bfloat16), dt_bias=dt0 + torch.log(-torch.expm1(-dt0)),
                A=-(0.5 + 15.5 * torch.rand(d_D, d_N, device=dev, generator=gen)), Dskip=torch.ones(d_D, device=dev),
                out_proj_w=(rn(d_dm, d_D) / d_D ** 0.5).to(torch.bfloat16))))
        drafter = MambaDrafter((0.5 * rn(d_V, d_dm)).to(torch.bfloat16), blocks_d, torch.ones(d_dm, device=dev))
        prefix = torch.randint(0, d_V, (d_L,), device=dev, generator=gen, dtype=torch.int32)

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            q0, q1 = ev(), ev()
            q0.record()
            for _ in range(reps):
                fn()
            q1.record()
            torch.cuda.synchronize()
            return q0.elapsed_time(q1) / reps
        drafter_detail = {"workload": "Mamba-130M-shaped drafter, %d blocks, d_model %d, vocabulary %d, random weights"
                                      % (d_nl, d_dm, d_V),
                          "prefill_%d_tokens_ms" % d_L: round(timed(lambda: drafter.prefill(prefix), 5), 4)}
        for name, tree in (("sequential_1_1_1_1_1", (1, 1, 1, 1, 1)), ("tree_3_2_2_1_1", (3, 2, 2, 1, 1)),
                           ("tree_2_2_2_1_1_1", (2, 2, 2, 1, 1, 1))):
            drafter.draft(tree)                                       # captures the round's graph
            drafter_detail[name + "_round_ms"] = round(timed(lambda: drafter.draft(tree), 20), 4)
        drafter_detail["per_position_us_sequential"] = round(drafter_detail["sequential_1_1_1_1_1_round_ms"] / 5 * 1e3, 1)
        drafter_detail["tree_over_sequential"] = round(drafter_detail["tree_3_2_2_1_1_round_ms"] /
                                                       drafter_detail["sequential_1_1_1_1_1_round_ms"], 3)
        del drafter, blocks_d

    # every synthetic config, one entry point at a time: median of many launches from HIP events on the
    # launch stream ("warm": same buffers every launch; "cold": a graph that walks rotating state
    # buffers of more than 512 MB, so that every launch streams its state from HBM)
    per_config = {}
    if args.all_configs:
        def median_ms(fn, n_warm=20, n=100):
            for _ in range(n_warm):
                fn()
            pairs = []
            for _ in range(n):
                q0, q1 = ev(), ev()
                q0.record()
                fn()
                q1.record()
                pairs.append((q0, q1))
            torch.cuda.synchronize()
            return float(np.median([a.elapsed_time(b) for a, b in pairs]))

        def graph_us(fn_round, launches, reps=5):
            fn_round()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            sd = torch.cuda.Stream()
            sd.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(sd):
                with torch.cuda.graph(g, stream=sd):
                    fn_round()
            torch.cuda.current_stream().wait_stream(sd)
            g.replay()
            q0, q1 = ev(), ev()
            q0.record()
            for _ in range(reps):
                g.replay()
            q1.record()
            torch.cuda.synchronize()
            return q0.elapsed_time(q1) * 1e3 / (reps * launches)

        rate = lambda nbytes, ms: {"GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                   "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                   "frac_of_copy_kernel": round(nbytes / (ms * 1e-3) / 1e9 / copy_gbs, 4)}
        for name in ("cfg0", "cfg1", "cfg3", "cfg4"):
            c = synth.CONFIGS[name]
            cB, cL, cD, cN, cK = c["batch"], c["L"], c["D"], c["N"], c["K"]
            ce = 2 if c["io"] == synth.BF16 else 4
            cs = synth.config_prefill(name)
            Q = {k: to_dev(cs[k]) for k in ("x", "z", "Bm", "Cm", "dt", "A", "Dskip", "dt_bias", "conv_w", "conv_bias")}
            del cs
            q_xc, q_out = torch.empty_like(Q["x"]), torch.empty_like(Q["x"])
            q_cs = torch.empty((cB, cD, cK - 1), dtype=Q["x"].dtype, device=dev)
            q_hf = torch.empty((cB, cD, cN), dtype=torch.float32, device=dev)
            q_ws = torch.empty(max(m.mamba_scan_workspace_bytes(cB, cL, cD, cN, 0), 16), dtype=torch.uint8, device=dev)
            n_l = 100 if name != "cfg4" else 30
            cms = median_ms(lambda: m.mamba_conv1d_fwd(Q["x"], Q["conv_w"], Q["conv_bias"], None, y=q_xc,
                                                       conv_state_out=q_cs), n=n_l)
            sms = median_ms(lambda: m.mamba_scan_fwd(q_xc, Q["dt"], Q["A"], Q["Bm"], Q["Cm"], Q["Dskip"], Q["z"],
                                                     Q["dt_bias"], out=q_out, h_final=q_hf, workspace=q_ws), n=n_l)
            ent = {"shape": "batch %d x L %d x D %d, N %d, K %d, %s I/O" % (cB, cL, cD, cN, cK, c["io"]),
                   "conv1d": dict(ms=round(cms, 5), tokens_per_s=round(cB * cL / (cms * 1e-3), 1),
                                  **rate(conv_bytes(cB, cL, cD, cK, ce), cms)),
                   "scan": dict(ms=round(sms, 5), tokens_per_s=round(cB * cL / (sms * 1e-3), 1),
                                TFLOPs=round(scan_flops(cB, cL, cD, cN) / (sms * 1e-3) / 1e12, 2),
                                frac_of_fp32_vector_peak=round(scan_flops(cB, cL, cD, cN) / (sms * 1e-3) / 1e12 /
                                                               FP32_VECTOR_PEAK_TFLOPS, 4),
                                **rate(scan_bytes(cB, cL, cD, cN, ce), sms)),
                   "timing": "median of %d launches (HIP events), launches below ~15 us are bound by the host" % n_l}
            per_config[name + "_prefill"] = ent
            del Q, q_xc, q_out, q_ws
        for name in ("cfg2", "cfg4"):
            c = synth.CONFIGS[name]
            cnb, cD, cN, cK, cnl = c["branches"], c["D"], c["N"], c["K"], c.get("n_layers", 1)
            ce = 2 if c["io"] == synth.BF16 else 4
            rg = np.random.default_rng(synth.SEEDS[name] + 500)
            lp = {k: to_dev(v) for k, v in synth.layer_params(rg, cD, cN, cK).items()}
            tk = {k: to_dev(v) for k, v in synth.token_inputs(rg, (cnb,), cD, cN, c["io"]).items()}
            par = to_dev(rg.integers(0, cnb, cnb).astype(np.int32))
            R = int(600e6 // (cnb * cD * cN * 4)) + 1
            hin = [torch.randn((cnb, cD, cN), device=dev) for _ in range(R)]
            hout = [torch.empty((cnb, cD, cN), device=dev) for _ in range(R)]
            cin = [torch.randn((cnb, cD, cK - 1), device=dev).to(tk["x"].dtype) for _ in range(R)]
            cout = [torch.empty_like(cin[0]) for _ in range(R)]
            so = torch.empty((cnb, cD), dtype=tk["x"].dtype, device=dev)
            sxc = torch.empty((cnb, 1, cD), dtype=tk["x"].dtype, device=dev)
            step_i = lambda i: m.mamba_state_step(hin[i], tk["x"], tk["dt"], lp["A"], tk["Bm"], tk["Cm"], lp["Dskip"],
                                                  tk["z"], lp["dt_bias"], parent_idx=par, h_out=hout[i], out=so)
            fork_i = lambda i: m.mamba_state_fork(cin[i].unsqueeze(0), hin[i].unsqueeze(0), par, conv_dst=cout[i].unsqueeze(0),
                                                  ssm_dst=hout[i].unsqueeze(0))
            conv_i = lambda i: m.mamba_conv1d_fwd(tk["x"].unsqueeze(1), lp["conv_w"], lp["conv_bias"],
                                                  conv_state_in=cout[i], y=sxc, conv_state_out=cout[i])
            full_i = lambda i: m.mamba_conv_state_step(hin[i], cin[i], tk["x"], lp["conv_w"], lp["conv_bias"], tk["dt"],
                                                       lp["A"], tk["Bm"], tk["Cm"], lp["Dskip"], tk["z"], lp["dt_bias"],
                                                       parent_idx=par, h_out=hout[i], conv_state_out=cout[i], out=so)
            sb_ = step_bytes(cnb, cD, cN, ce)
            fb_ = cnb * 2 * (cD * cN * 4 + cD * (cK - 1) * ce)
            cb_ = cnb * (2 * cD * (cK - 1) * ce + 2 * cD * ce)
            ent = {"shape": "%d branches, D %d, N %d, K %d, %s I/O, one layer; %d rotating buffer sets" %
                            (cnb, cD, cN, cK, c["io"], R)}
            for label, fn_i, nbytes in (("state_step_fused_parent", step_i, sb_), ("state_fork_unfused", fork_i, fb_),
                                        ("conv_step", conv_i, cb_),
                                        ("fork_conv_step_state_step_one_launch", full_i, sb_ + cnb * 2 * cD * (cK - 1) * ce)):
                cold = graph_us(lambda: [fn_i(i) for i in range(R)], R)
                warm = graph_us(lambda: [fn_i(0) for _ in range(R)], R)
                ent[label] = {"algorithmic_bytes": nbytes, "cold_us": round(cold, 3), "warm_us": round(warm, 3),
                              "cold": rate(nbytes, cold * 1e-3), "warm": rate(nbytes, warm * 1e-3),
                              "branch_steps_per_s_per_layer_cold": round(cnb / (cold * 1e-6), 1)}
            ent["timing"] = "per launch inside a replayed HIP graph of %d launches" % R
            per_config[name + "_decode"] = ent
            del hin, hout, cin, cout

    # the scalar-decay (Mamba-2 style) core at Mamba2-130M-like shapes: 24 heads x 64 channels, 128 states
    ssd_detail = {}
    if not args.no_mamba2:
        sH, sP, sN = 24, 64, 128
        gen2 = torch.Generator(device=dev)
        gen2.manual_seed(222)
        rn2 = lambda *shape: torch.randn(*shape, device=dev, generator=gen2)
        sA = -(0.05 + 1.45 * torch.rand(sH, device=dev, generator=gen2))
        sD, sb_ = torch.ones(sH, device=dev), torch.full((sH,), -2.5, device=dev)
        ssd_detail = {"workload": "%d heads x %d channels, %d states, one group, bf16 I/O" % (sH, sP, sN)}
        for sL in (2048, 32768):
            sx, sz = rn2(1, sL, sH, sP).to(torch.bfloat16), rn2(1, sL, sH, sP).to(torch.bfloat16)
            sdt = (0.5 * rn2(1, sL, sH)).to(torch.bfloat16)
            sB, sC = rn2(1, sL, sN).to(torch.bfloat16), rn2(1, sL, sN).to(torch.bfloat16)
            so, sh = torch.empty_like(sx), torch.empty((1, sH, sP, sN), device=dev)
            sws = torch.empty(m.mamba2_ssd_workspace_bytes(1, sL, sH, sP, sN), dtype=torch.uint8, device=dev)
            run_ssd = lambda: m.mamba2_ssd_fwd(sx, sdt, sA, sB, sC, sD, sz, sb_, None, out=so, h_final=sh, workspace=sws)
            for _ in range(3):
                run_ssd()
            q0, q1 = ev(), ev()
            q0.record()
            for _ in range(10):
                run_ssd()
            q1.record()
            torch.cuda.synchronize()
            s_ms = q0.elapsed_time(q1) / 10
            s_bytes = sL * (3 * sH * sP + 2 * sN + sH) * 2
            ssd_detail["scan_L%d" % sL] = {"ms": round(s_ms, 4), "tokens_per_s": round(sL / (s_ms * 1e-3), 1),
                                           "algorithmic_GBps": round(s_bytes / (s_ms * 1e-3) / 1e9, 1)}
            del sx, sz, sdt, sB, sC, so, sws
        snb = 64
        Rs = 12
        shin = [rn2(snb, sH, sP, sN) for _ in range(Rs)]
        shout = [torch.empty_like(shin[0]) for _ in range(Rs)]
        tx, tz = rn2(snb, sH, sP).to(torch.bfloat16), rn2(snb, sH, sP).to(torch.bfloat16)
        tdt, tB, tC = rn2(snb, sH).to(torch.bfloat16), rn2(snb, sN).to(torch.bfloat16), rn2(snb, sN).to(torch.bfloat16)
        tpar = torch.randint(0, snb, (snb,), device=dev, dtype=torch.int32, generator=gen2)
        tout = torch.empty_like(tx)

        def ssd_round():
            for i in range(Rs):
                m.mamba2_state_step(shin[i], tx, tdt, sA, tB, tC, sD, tz, sb_, parent_idx=tpar, h_out=shout[i], out=tout)
        ssd_round()
        torch.cuda.synchronize()
        sg = torch.cuda.CUDAGraph()
        side3 = torch.cuda.Stream()
        side3.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side3):
            with torch.cuda.graph(sg, stream=side3):
                ssd_round()
        torch.cuda.current_stream().wait_stream(side3)
        sg.replay()
        q0, q1 = ev(), ev()
        q0.record()
        for _ in range(5):
            sg.replay()
        q1.record()
        torch.cuda.synchronize()
        s_us = q0.elapsed_time(q1) * 1e3 / (5 * Rs)
        st_bytes = snb * (2 * sH * sP * sN * 4 + (3 * sH * sP + 2 * sN + sH) * 2)
        ssd_detail["state_step_%d_branches" % snb] = {
            "us_per_launch": round(s_us, 3), "algorithmic_bytes_per_launch": st_bytes,
            "GBps": round(st_bytes / s_us / 1e3, 1), "frac_of_hbm_peak": round(st_bytes / s_us / 1e3 / HBM_PEAK_GBS, 4),
            "frac_of_copy_kernel": round(st_bytes / s_us / 1e3 / copy_gbs, 4),
            "timing": "per launch in a replayed HIP graph over %d rotating state sets (%.0f MB)" % (Rs, Rs * 2 * snb * sH * sP * sN * 4 / 1e6)}
        del shin, shout

    tokens = B * L
    sb = scan_bytes(B, L, D, N, e)
    achieved = sb / (scan_ms * 1e-3) / 1e9
    tflops = scan_flops(B, L, D, N) / (scan_ms * 1e-3) / 1e12
    choice = {"chunked": "scan_chunk_state + scan_carry + scan_chunk_out: time chunks across workgroups",
              "single": "scan_chunk_out: a single chunk", "direct": "scan_direct_kernel: one pass, channels across lanes",
              "lanes": "scan_lanes_kernel: one pass, time across lanes"}
    roofline = {
        "kernel": "mamba_scan_fwd (%s)" % choice[m.mamba_scan_kernel(B, L, D, N)],
        "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": scan_traffic_bytes(args.prefill),
        "algorithmic_bytes_per_launch": sb, "avg_launch_ms": round(scan_ms, 5),
        "frac_of_copy_kernel": round(achieved / copy_gbs, 4),
        "binding_resource": "vector ALU: one exp2 and four plain fp32 instructions per state update",
        "alu": {"achieved": round(tflops, 2), "unit": "TFLOP/s", "algorithmic_flops_per_launch": scan_flops(B, L, D, N),
                "peak_published_fp32_vector": FP32_VECTOR_PEAK_TFLOPS, "frac_of_published": round(tflops / FP32_VECTOR_PEAK_TFLOPS, 4),
                "peak_without_packed_fp32": FP32_VECTOR_PLAIN_TFLOPS, "frac_without_packed_fp32": round(tflops / FP32_VECTOR_PLAIN_TFLOPS, 4)},
    }
    units = nb * nsteps * nl
    if args.staged_decode:
        # state step + conv step (window in and out, x in, x_c out) + conv-state fork (window in and out)
        dec_bytes = nsteps * nl * (step_bytes(nb, Dd, Nd, ed) + nb * (2 * Dd * (Kd - 1) * ed + 2 * Dd * ed)) \
            + nsteps * nl * nb * 2 * Dd * (Kd - 1) * ed
    else:
        # one launch: the state step's bytes (its x is the input before the conv) + the window in and out
        dec_bytes = nsteps * nl * (step_bytes(nb, Dd, Nd, ed) + nb * 2 * Dd * (Kd - 1) * ed)
    detail = {
        "prefill_conv_ms": round(conv_ms, 5), "prefill_scan_ms": round(scan_ms, 5),
        "prefill_tokens_per_s": round(tokens / ((conv_ms + scan_ms) * 1e-3), 1),
        "scan_tokens_per_s": round(tokens / (scan_ms * 1e-3), 1),
        "conv_GBps": round(conv_bytes(B, L, D, K, e) / (conv_ms * 1e-3) / 1e9, 1),
        "decode_ms": round(dec_ms, 5),
        "decode_branch_steps_per_s_per_layer": round(units / (dec_ms * 1e-3), 1),
        "decode_GBps": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1),
        "decode_launches": nsteps * (1 + 2 * nl) if args.staged_decode else nsteps * nl,
        "decode_stages": "fork + conv step + state step" if args.staged_decode else "one launch per layer and step (mamba_conv_state_step)", "decode_mode": "eager" if args.eager_decode else "hip_graph",
        "copy_kernel_GBps": round(copy_gbs, 1), "wide_decode_step": wide, "scan_other_shapes": other_scans,
        "tree_draft_round": tree_detail, "whole_block": block_detail,
        "whole_drafter": drafter_detail, "mamba2_core": ssd_detail, "per_config": per_config,
    }

    result = {
        "metric": "scan prefill tokens/s + %HBM peak; tree-decode branch-steps/s per layer",
        "value": round(tokens / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s prefill (conv1d+scan, batch %d x L=%d, D=%d, N=%d, %s I/O) + %s tree "
                               "decode (%d layers x %d branches x %d draft steps, fork+conv step+state step%s)"
                               % (args.prefill, B, L, D, N, pc["io"], args.decode, nl, nb, nsteps, "" if args.staged_decode else " in one launch per layer"),
                   "io_dtype": pc["io"], "state_dtype": "f32"},
        "roofline": roofline, "detail": detail,
    }

    if not args.no_cpu_baseline:
        import oracle
        W = lambda a: oracle.widen(a, bf16=(a.dtype == np.uint16))
        ox = {k: W(case[k]) for k in ("x", "z", "Bm", "Cm", "dt", "A", "Dskip", "dt_bias", "conv_w",
                                      "conv_bias")}
        reps = 3
        c0 = time.perf_counter()
        for _ in range(reps):
            rxc, _ = oracle.conv1d_fwd(ox["x"], ox["conv_w"], ox["conv_bias"])
            oracle.scan_fwd(rxc, ox["dt"], ox["A"], ox["Bm"], ox["Cm"], ox["Dskip"], ox["z"], ox["dt_bias"])
        c1 = time.perf_counter()
        sec = (c1 - c0) / reps
        result["cpu_baseline"] = {
            "value": round(tokens / sec, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "%s prefill leg only (conv1d + scan, all %d channels, %d tokens), fp64, mean of "
                      "%d runs of %.2f s wall (%.0f core-seconds in all)"
                      % (args.prefill, D, tokens, reps, sec, reps * sec * oracle.num_threads())}
        if args.all_configs:
            # the oracle on every config, all threads; one thread as well where that takes seconds
            per = {}
            for name in ("cfg0", "cfg1", "cfg3", "cfg4"):
                c = synth.CONFIGS[name]
                cs = synth.config_prefill(name)
                oq = {k: W(cs[k]) for k in ("x", "z", "Bm", "Cm", "dt", "A", "Dskip", "dt_bias", "conv_w", "conv_bias")}
                del cs

                def run_oracle():
                    q0 = time.perf_counter()
                    rx, _ = oracle.conv1d_fwd(oq["x"], oq["conv_w"], oq["conv_bias"])
                    q1 = time.perf_counter()
                    oracle.scan_fwd(rx, oq["dt"], oq["A"], oq["Bm"], oq["Cm"], oq["Dskip"], oq["z"], oq["dt_bias"])
                    return q1 - q0, time.perf_counter() - q1
                tc, ts = run_oracle()
                ntok = c["batch"] * c["L"]
                name = name + "_prefill"
                per[name] = {"threads": oracle.num_threads(), "conv1d_s": round(tc, 4), "scan_s": round(ts, 4),
                             "scan_tokens_per_s": round(ntok / ts, 1), "prefill_tokens_per_s": round(ntok / (tc + ts), 1)}
                if name in ("cfg0_prefill", "cfg1_prefill"):
                    oracle.set_num_threads(1)
                    tc1, ts1 = run_oracle()
                    oracle.set_num_threads(per[name]["threads"])
                    per[name]["one_thread"] = {"conv1d_s": round(tc1, 4), "scan_s": round(ts1, 4),
                                               "scan_tokens_per_s": round(ntok / ts1, 1)}
                del oq
            for name in ("cfg2", "cfg4"):
                c = synth.CONFIGS[name]
                rg = np.random.default_rng(synth.SEEDS[name] + 500)
                lp = {k: W(v) for k, v in synth.layer_params(rg, c["D"], c["N"], c["K"]).items()}
                tk = {k: W(v) for k, v in synth.token_inputs(rg, (c["branches"],), c["D"], c["N"], c["io"]).items()}
                par = rg.integers(0, c["branches"], c["branches"]).astype(np.int32)
                h_in = rg.standard_normal((c["branches"], c["D"], c["N"]))
                reps_o = 20
                q0 = time.perf_counter()
                for _ in range(reps_o):
                    oracle.state_step(h_in, tk["x"], tk["dt"], lp["A"], tk["Bm"], tk["Cm"], lp["Dskip"], tk["z"],
                                      lp["dt_bias"], parent=par)
                sec_o = (time.perf_counter() - q0) / reps_o
                per[name + "_decode"] = {"threads": oracle.num_threads(), "state_step_s": round(sec_o, 6),
                             "branch_steps_per_s_per_layer": round(c["branches"] / sec_o, 1)}
            result["cpu_baseline"]["per_config"] = per
    print(json.dumps(result))


if __name__ == "__main__":
    main()
