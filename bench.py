"""Benchmark of the LSM chunkwise forward+backward on one MI355X.

A step = one lsm_chunk_fwd + one lsm_chunk_bwd over one batch of synthetic inputs of the chosen
benchmark configuration (default: configuration 3, the shape the headline metric is quoted on:
B=4, H=16, T=8192, d_k=d_v=128, per-token scalar decay, bf16, chunk 64).  Inputs, outputs and the
workspace are resident in HBM before the timed region starts.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def algorithmic_bytes_per_token_head(cfg, which):
    """Compulsory HBM bytes per token-head: every input read once, every output written once."""
    e = 2 if cfg["dtype"] == "bf16" else 4
    dk, dv = cfg["dk"], cfg["dv"]
    gam = {0: 0, 1: 0, 2: 4, 3: 4 * dk}[cfg["kind"]]
    fwd = (2 * dk + dv) * e + gam + dv * e
    bwd = (2 * dk + 2 * dv) * e + gam + (2 * dk + dv) * e + gam
    return {"fwd": fwd, "bwd": bwd, "both": fwd + bwd}[which]


def algorithmic_flops_per_token_head(cfg):
    """Chunk-dense convention: the full C x C block is computed and masked (Algorithm 2)."""
    dk, dv, C = cfg["dk"], cfg["dv"], cfg["chunk"]
    fwd = 2 * C * (dk + dv) + 4 * dk * dv
    bwd = 2 * C * (3 * dk + 2 * dv) + 8 * dk * dv
    return fwd, bwd


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration 1..5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--layout", type=int, default=0, choices=(0, 1),
                    help="0: [B,H,T,d] as BASELINE.json's configurations are written; 1: the same data token-major [B,T,H,d]")
    ap.add_argument("--states", choices=("recompute", "saved"), default="saved",
                    help="chunk states of the backward pass: kept by the forward call in the shared workspace (where "
                         "the library finds that faster), or computed again from the inputs; the other mode is timed "
                         "too and reported beside the headline")
    ap.add_argument("--no-microbench", action="store_true",
                    help="skip the LDS-resident intra-chunk micro-benchmark (profiling runs: it launches the output kernel again)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import lsm_workloads as wl
    import paper_2503_05447_amd as pkg

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    x, cfg = wl.make_config(args.config - 1)
    backward = cfg["backward"]
    tdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32

    def mv(a, dt):
        return None if a is None else torch.from_numpy(a).to(dev).to(dt).contiguous()

    q, k, v, d_o = (mv(x[n], tdt) for n in ("q", "k", "v", "d_o"))
    g, m0 = mv(x["g"], torch.float32), mv(x["m0"], torch.float32)
    kind, C = cfg["kind"], cfg["chunk"]
    B, H, T, dk, dv = cfg["B"], cfg["H"], cfg["T"], cfg["dk"], cfg["dv"]
    saved = args.states == "saved"
    p = pkg.make_params(B, H, T, dk, dv, C, kind, 1 if cfg["dtype"] == "bf16" else 0,
                        flags=pkg.FLAG_SAVE_STATES if saved else 0)
    p_keep = pkg.make_params(B, H, T, dk, dv, C, kind, 1 if cfg["dtype"] == "bf16" else 0, flags=pkg.FLAG_SAVE_STATES)
    ws = torch.empty(max(pkg.lsm_chunk_fwd_workspace_bytes(p), pkg.lsm_chunk_bwd_workspace_bytes(p),
                         pkg.lsm_chunk_fwd_workspace_bytes(p_keep), 256), dtype=torch.uint8, device=dev)
    # what the library does with the request (it recomputes where keeping the states would be slower)
    kept = {True: "saved by the forward call", False: "recomputed"}

    if args.layout == 1:   # the same values, token-major
        q, k, v, d_o = (t_.transpose(1, 2).contiguous() for t_ in (q, k, v, d_o))
        if kind in (wl.KIND_SCALAR, wl.KIND_VECTOR):
            g = g.transpose(1, 2).contiguous()

    def step(saved=saved):
        out = pkg.lsm_chunk_fwd(q, k, v, g, kind, C, m0, workspace=ws, layout=args.layout, save_states=saved)
        grads = pkg.lsm_chunk_bwd(q, k, v, g, kind, d_o, C, m0, workspace=ws, layout=args.layout,
                                  states_saved=saved) if backward else None
        return out, grads

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        last = step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec = (t1 - t0) / args.steps
    # Per-kernel durations: the same K steps once more with a pair of HIP events around every launch, on
    # the launch stream.  The events keep consecutive kernels from overlapping and cost several percent of
    # a step, so this pass is timed on its own (ms_per_step_with_events) and not reported as the throughput.
    pkg.lsm_profile_start()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec_events = (time.perf_counter() - t2) / args.steps
    prof = pkg.lsm_profile_stop()
    tokens = B * T
    th = B * H * T

    per_kernel = {}
    for name, ms in prof:
        per_kernel.setdefault(name, []).append(ms)
    kavg = {n: float(np.mean(v_)) for n, v_ in per_kernel.items()}
    dominant = max(kavg, key=kavg.get)
    # algorithmic bytes of the dominant kernel's launch: the compulsory traffic of the pass it belongs to
    which = "bwd" if ("grad" in dominant or "bwd" in dominant or "dstate" in dominant) else "fwd"
    abytes = algorithmic_bytes_per_token_head(cfg, which) * th
    achieved = abytes / (kavg[dominant] * 1e-3) / 1e9
    ffl, bfl = algorithmic_flops_per_token_head(cfg)
    flops = (ffl + (bfl if backward else 0)) * th
    tflops = flops / sec / 1e12

    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            key = cfg["name"] + ("" if pkg.keeps_states(p) == 1 else "_recompute")
            traffic = json.load(f).get(key, {}).get(dominant)
    except (OSError, ValueError):
        pass

    result = {
        "metric": "LSM chunkwise fwd+bwd tokens/s and TFLOP/s (%MFMA peak) at H=16,d=128,T=8192",
        "value": tokens / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": cfg["name"], "B": B, "H": H, "T": T, "d_k": dk, "d_v": dv, "chunk": C,
                   "decay_kind": wl.KIND_NAMES[kind], "passes": "fwd+bwd" if backward else "fwd",
                   "kernel_path": "mfma" if pkg.kernel_path(p) == 1 else "generic",
                   "layout": "BTHD" if args.layout else "BHTD", "bwd_states": kept[pkg.keeps_states(p) == 1]},
        "tflops": tflops, "mfma_peak_frac": tflops / MFMA_BF16_PEAK_TFLOPS,
        "hbm_frac_whole_step": algorithmic_bytes_per_token_head(cfg, "both" if backward else "fwd") * th / sec / 1e9 / HBM_PEAK_GBS,
        "kernel_ms": kavg, "ms_per_step_with_events": sec_events * 1e3,
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": abytes},
    }

    if backward and not args.no_microbench:   # the same steps with the other treatment of the chunk states
        for _ in range(args.warmup):
            step(not saved)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(not saved)
        torch.cuda.synchronize()
        sec2 = (time.perf_counter() - t0) / args.steps
        other = kept[False] if saved else kept[pkg.keeps_states(p_keep) == 1]
        result["other_bwd_states"] = {"bwd_states": other, "ms_per_step": sec2 * 1e3, "value": tokens / sec2,
                                      "unit": "tokens/s"}

    if pkg.kernel_path(p) == 1 and kind != wl.KIND_VECTOR and not args.no_microbench and args.layout == 0:
        # Intra-chunk phase apart from HBM: the forward per-chunk kernel with its compute phase repeated on
        # LDS-resident tiles; the time of one pass is the slope between two repeat counts.
        R = 33
        o_mb = torch.empty_like(last[0][0])
        o_plain, _ = pkg.lsm_chunk_fwd(q, k, v, g, kind, C, None, workspace=ws)
        ws_mb = pkg.lsm_bench_intra_chunk_workspace(q, k, v, g, kind, C)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        pkg.lsm_bench_intra_chunk(q, k, v, g, kind, o_mb, ws_mb, 1, C)
        ev[0].record(); pkg.lsm_bench_intra_chunk(q, k, v, g, kind, o_mb, ws_mb, 1, C); ev[1].record()
        ev[2].record(); pkg.lsm_bench_intra_chunk(q, k, v, g, kind, o_mb, ws_mb, R, C); ev[3].record()
        torch.cuda.synchronize()
        t1_ms, tR_ms = ev[0].elapsed_time(ev[1]), ev[2].elapsed_time(ev[3])
        pass_s = (tR_ms - t1_ms) / (R - 1) * 1e-3
        chunks = B * H * ((T + C - 1) // C)
        alg = chunks * (2 * C * C * (dk + dv) + 2 * C * dk * dv)          # dense C x C block + Q S_c (Algorithm 2)
        # issued MFMA 32x32x16 per chunk: Q S_c 4 x 16, three score blocks x 8, A V with head + remainder 4 x 12
        issued = chunks * 136 * 2 * 32 * 32 * 16
        result["intra_chunk_microbench"] = {
            "what": "forward per-chunk kernel (scores, mask/decay, A V, Q S_c), compute phase repeated on LDS-resident tiles",
            "repeats": R, "ms_one_pass": pass_s * 1e3, "ms_streamed_kernel": t1_ms,
            "algorithmic_tflops": alg / pass_s / 1e12, "algorithmic_frac_of_mfma_peak": alg / pass_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "issued_mfma_tflops": issued / pass_s / 1e12, "issued_frac_of_mfma_peak": issued / pass_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "max_abs_diff_to_forward": float((o_mb.float() - o_plain.float()).abs().max())}
        try:   # the matrix-pipe utilisation the hardware counters give for the same launches (collected under rocprofv3)
            with open(os.path.join(ROOT, "profiles", "mfma_counters.json")) as f:
                result["intra_chunk_microbench"]["rocprof_counters"] = json.load(f).get(cfg["name"] + "_intra_chunk_microbench")
        except (OSError, ValueError):
            pass

    if not args.no_microbench:
        # Recurrent decoding step (lsm_step) on the heads of this workload: state read + written once per step.
        dec = {}
        for Bd in (16, 256):
            qd = torch.randn(Bd, H, dk, device=dev).to(tdt)
            kd = torch.randn(Bd, H, dk, device=dev).to(tdt) / dk ** 0.5
            vd = torch.randn(Bd, H, dv, device=dev).to(tdt)
            gd = {wl.KIND_NONE: None, wl.KIND_HEAD: g}.get(kind, None)
            if kind == wl.KIND_SCALAR:
                gd = -torch.rand(Bd, H, device=dev)
            elif kind == wl.KIND_VECTOR:
                gd = -torch.rand(Bd, H, dk, device=dev)
            st = torch.zeros(Bd, H, dk, dv, device=dev)
            od = torch.empty(Bd, H, dv, device=dev, dtype=tdt)
            nst = 200
            for _ in range(20):
                pkg.lsm_step(qd, kd, vd, gd, kind, st, od)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(nst):
                pkg.lsm_step(qd, kd, vd, gd, kind, st, od)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / nst
            # the same loop recorded once into a HIP graph and replayed: no per-step launch cost on the host
            gsteps, greps = 50, 8
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(gsteps):
                    pkg.lsm_step(qd, kd, vd, gd, kind, st, od)
            graph.replay()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(greps):
                graph.replay()
            e1.record()
            torch.cuda.synchronize()
            us_g = e0.elapsed_time(e1) * 1e3 / (gsteps * greps)
            state_bytes = Bd * H * dk * dv * 8
            dec["batch_%d" % Bd] = {"us_per_step": us, "us_per_step_graph_replay": us_g, "tokens_per_s": Bd / (min(us, us_g) * 1e-6),
                                    "state_GBps": state_bytes / (min(us, us_g) * 1e-6) / 1e9, "state_bytes_per_step": state_bytes}
        result["decode_step"] = {"what": "lsm_step, one token per sequence, H=%d d_k=%d d_v=%d, back-to-back launches on one stream "
                                         "(launch overhead included); state_GBps = fp32 state read + written per step" % (H, dk, dv),
                                 **dec}

    if not args.no_cpu_baseline or not args.no_check:
        from oracle import lsm_oracle_bwd, lsm_oracle_fwd, oracle_threads
        # bounded sample: the first `nb` batch elements of the same workload (all heads, full T)
        nb = max(1, min(B, (1 << 20) // (H * T) or 1))
        sl = slice(0, nb)
        gs = x["g"] if (x["g"] is None or kind == wl.KIND_HEAD) else x["g"][sl]
        m0s = None if x["m0"] is None else x["m0"][sl]
        c0 = time.perf_counter()
        o_ref, mT_ref = lsm_oracle_fwd(x["q"][sl], x["k"][sl], x["v"][sl], gs, kind, m0s)
        r_ref = lsm_oracle_bwd(x["q"][sl], x["k"][sl], x["v"][sl], gs, kind, x["d_o"][sl], m0s) if backward else None
        c1 = time.perf_counter()
        result["cpu_baseline"] = {"value": nb * T / (c1 - c0), "unit": "tokens/s", "cores": oracle_threads(),
                                  "kind": "oracle",
                                  "sample": "batch elements 0..%d of the same workload, all %d heads, full T=%d, %s"
                                            % (nb - 1, H, T, "fwd+bwd" if backward else "fwd"),
                                  "seconds": c1 - c0}
        if not args.no_check:
            (o, mT), grads = last
            if args.layout == 1:   # back to the order of the oracle's arrays
                o = o.transpose(1, 2)
                if grads:
                    grads = {n_: (t_.transpose(1, 2) if (t_ is not None and t_.dim() >= 3 and n_ != "d_init_state") else t_)
                             for n_, t_ in grads.items()}
            def err(got, ref, ulp):
                got = got.float().cpu().numpy().astype(np.float64)
                e = np.maximum(np.abs(got - ref) - ulp * np.abs(ref), 0).max()
                return float(e / max(np.sqrt(np.mean(ref ** 2)), 1e-300))
            ulp = 2.0 ** -8 if cfg["dtype"] == "bf16" else 0.0   # half-ulp of the bf16 output container
            par = {"o": err(o[sl], o_ref, ulp), "final_state": err(mT[sl], mT_ref, 0.0)}
            if backward:
                par.update(dq=err(grads["dq"][sl], r_ref["dq"], ulp), dk=err(grads["dk"][sl], r_ref["dk"], ulp),
                           dv=err(grads["dv"][sl], r_ref["dv"], ulp))
                if kind in (wl.KIND_SCALAR, wl.KIND_VECTOR):
                    par["dg"] = err(grads["dg"][sl], r_ref["dg"], 0.0)
            result["parity_err_over_rms"] = par
    print(json.dumps(result))


if __name__ == "__main__":
    main()
