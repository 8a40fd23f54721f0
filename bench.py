#!/usr/bin/env python3
"""Benchmark of the selective-SSM layer core on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
  prefill  conv1d + selective scan over the long context (Mamba-130M-shaped layer, batch 1,
           L = 32768 tokens, bf16 I/O, fp32 state), then
  decode   tree drafting over 24 such layers: 5 draft steps of 32 live branches; per draft step
           one conv-state fork for all layers, and per layer a conv step and a state step with
           the SSM-state fork fused in (parent index).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

The roofline object covers the dominant call, the selective scan: algorithmic bytes per launch
(x, dt, z, out, B, C; nothing else) over its average duration, measured with HIP events on the
launch stream inside the timed region, against the 8 TB/s HBM peak.  The oracle (fp64, CPU) is
timed on the same prefill for cpu_baseline.
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
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector, published (needs packed fp32)


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
    """fp32 operations of the scan as defined: per state update delta*A, exp, (delta x)*B, fma, fma
    = 7; per (token, channel) softplus, skip, gate and products ~ 16."""
    return B * L * D * (7 * N + 16)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run three plain 1 GiB device copies: the known-size "
                         "reference that the FETCH_SIZE / WRITE_SIZE counters are scaled by")
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
    ssm = [to_dev(dc["ssm0"]), torch.empty((nl, nb, Dd, Nd), dtype=torch.float32, device=dev)]
    conv = [to_dev(dc["conv0"]), torch.empty_like(to_dev(dc["conv0"]))]
    dxc = torch.empty((nb, 1, Dd), dtype=conv[0].dtype, device=dev)
    dout = torch.empty((nb, Dd), dtype=conv[0].dtype, device=dev)

    def prefill():
        m.mamba_conv1d_fwd(P["x"], P["conv_w"], P["conv_bias"], None, y=xc, conv_state_out=conv_state)
        m.mamba_scan_fwd(xc, P["dt"], P["A"], P["Bm"], P["Cm"], P["Dskip"], P["z"], P["dt_bias"],
                         out=out, h_final=h_final, workspace=ws)

    def decode():
        cur = 0
        for s in range(nsteps):
            nxt = 1 - cur
            m.mamba_state_fork(conv[cur], None, PAR[s], conv_dst=conv[nxt])
            for l in range(nl):
                t = TOK[s][l]
                m.mamba_conv1d_fwd(t["x"].unsqueeze(1), LP[l]["conv_w"], LP[l]["conv_bias"],
                                   conv_state_in=conv[nxt][l], y=dxc, conv_state_out=conv[nxt][l])
                m.mamba_state_step(ssm[cur][l], dxc.squeeze(1), t["dt"], LP[l]["A"], t["Bm"], t["Cm"],
                                   LP[l]["Dskip"], t["z"], LP[l]["dt_bias"], parent_idx=PAR[s],
                                   h_out=ssm[nxt][l], out=dout)
            cur = nxt

    ev = lambda: torch.cuda.Event(enable_timing=True)
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

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    tokens = B * L
    sb = scan_bytes(B, L, D, N, e)
    achieved = sb / (scan_ms * 1e-3) / 1e9
    roofline = {
        "kernel": "mamba_scan_fwd (scan_chunk_state + scan_carry + scan_chunk_out)",
        "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
        "algorithmic_bytes_per_launch": sb, "avg_launch_ms": round(scan_ms, 5),
        "alu": {"achieved_tflops": round(scan_flops(B, L, D, N) / (scan_ms * 1e-3) / 1e12, 2),
                "peak_tflops": FP32_VECTOR_PEAK_TFLOPS,
                "frac": round(scan_flops(B, L, D, N) / (scan_ms * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS, 4)},
    }
    units = nb * nsteps * nl
    dec_bytes = nsteps * nl * (step_bytes(nb, Dd, Nd, ed) + nb * (2 * Dd * (Kd - 1) * ed + 2 * Dd * ed)) \
        + nsteps * nl * nb * 2 * Dd * (Kd - 1) * ed
    detail = {
        "prefill_conv_ms": round(conv_ms, 5), "prefill_scan_ms": round(scan_ms, 5),
        "prefill_tokens_per_s": round(tokens / ((conv_ms + scan_ms) * 1e-3), 1),
        "scan_tokens_per_s": round(tokens / (scan_ms * 1e-3), 1),
        "conv_GBps": round(conv_bytes(B, L, D, K, e) / (conv_ms * 1e-3) / 1e9, 1),
        "decode_ms": round(dec_ms, 5),
        "decode_branch_steps_per_s_per_layer": round(units / (dec_ms * 1e-3), 1),
        "decode_GBps": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1),
        "decode_launches": nsteps * (1 + 2 * nl),
    }

    result = {
        "metric": "scan prefill tokens/s + %HBM peak; tree-decode branch-steps/s per layer",
        "value": round(tokens / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s prefill (conv1d+scan, batch %d x L=%d, D=%d, N=%d, %s I/O) + %s tree "
                               "decode (%d layers x %d branches x %d draft steps, fork+conv step+state step)"
                               % (args.prefill, B, L, D, N, pc["io"], args.decode, nl, nb, nsteps),
                   "io_dtype": pc["io"], "state_dtype": "f32"},
        "roofline": roofline, "detail": detail,
    }

    if not args.no_cpu_baseline:
        import oracle
        W = lambda a: oracle.widen(a, bf16=(a.dtype == np.uint16))
        ox = {k: W(case[k]) for k in ("x", "z", "Bm", "Cm", "dt", "A", "Dskip", "dt_bias", "conv_w",
                                      "conv_bias")}
        c0 = time.perf_counter()
        rxc, _ = oracle.conv1d_fwd(ox["x"], ox["conv_w"], ox["conv_bias"])
        oracle.scan_fwd(rxc, ox["dt"], ox["A"], ox["Bm"], ox["Cm"], ox["Dskip"], ox["z"], ox["dt_bias"])
        c1 = time.perf_counter()
        result["cpu_baseline"] = {
            "value": round(tokens / (c1 - c0), 1), "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "%s prefill leg only (conv1d + scan, all %d channels, %d tokens), fp64, one run, "
                      "%.1f s" % (args.prefill, D, tokens, c1 - c0)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
