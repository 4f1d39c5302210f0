"""Benchmark of the LSM chunkwise forward+backward on one MI355X.

A step = one lsm_chunk_fwd + one lsm_chunk_bwd over one batch of synthetic inputs of the chosen
benchmark configuration (default: configuration 3, the shape the headline metric is quoted on:
B=4, H=16, T=8192, d_k=d_v=128, per-token scalar decay, bf16, chunk 64).  Inputs, outputs and the
workspace are resident in HBM before the timed region starts.  Prints ONE JSON line, which also
carries the other four configurations (`all_configs`), the roofline of the dominant kernel, the
calibrated peaks of this GPU and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
BF16_HALF_ULP = 2.0 ** -8       # half an ulp of a bf16 number relative to its magnitude (upper bound)


def algorithmic_bytes_per_token_head(cfg, which):
    """Compulsory HBM bytes per token-head: every input read once, every output written once."""
    e = 2 if cfg["dtype"] == "bf16" else 4
    dk, dv = cfg["dk"], cfg["dv"]
    gam = {0: 0, 1: 0, 2: 4, 3: 4 * dk}[cfg["kind"]]
    fwd = (2 * dk + dv) * e + gam + dv * e
    bwd = (2 * dk + 2 * dv) * e + gam + (2 * dk + dv) * e + gam
    return {"fwd": fwd, "bwd": bwd, "both": fwd + bwd}[which]


def algorithmic_flops_per_token_head(cfg, causal_exact=False):
    """Chunk-dense convention: the full C x C block is computed and masked (Algorithm 2).
    causal_exact: only the pairs r <= j of a chunk are counted (2C -> C + 1)."""
    dk, dv, C = cfg["dk"], cfg["dv"], cfg["chunk"]
    cc = (C + 1) if causal_exact else 2 * C
    fwd = cc * (dk + dv) + 4 * dk * dv
    bwd = cc * (3 * dk + 2 * dv) + 8 * dk * dv
    return fwd, bwd


# Which of the caller's tensors a kernel reads and writes: "fwd" / "bwd" = the whole compulsory traffic of
# that pass (the kernel reads every input and writes every output of it once); None = the kernel produces
# no output of the method (summaries, scans, tables: overhead of the chunkwise scheme), so no roofline
# fraction is quoted for it.
KERNEL_PASS = {
    "walk_fwd": "fwd", "walk_grad": "bwd",
    "mfma_output": "fwd", "mfma_grad": "bwd",          # vector kind: per-chunk kernels
    "generic_output": "fwd", "generic_grad": "bwd",
}


def rel_err(got, ref, ulp):
    import numpy as np
    e = float(np.maximum(np.abs(got - ref) - ulp * np.abs(ref), 0).max())
    rms = float(np.sqrt(np.mean(ref ** 2)))
    return e / rms if rms > 0 else e


class Workload:
    """One benchmark configuration resident on the GPU."""

    def __init__(self, index, layout=0, saved=True):
        import torch
        import lsm_workloads as wl
        import paper_2503_05447_amd as pkg
        self.pkg, self.torch, self.wl = pkg, torch, wl
        self.x, self.cfg = wl.make_config(index - 1)
        cfg = self.cfg
        dev = torch.device("cuda:0")
        tdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        mv = lambda a, dt: None if a is None else torch.from_numpy(a).to(dev).to(dt).contiguous()
        self.q, self.k, self.v, self.d_o = (mv(self.x[n], tdt) for n in ("q", "k", "v", "d_o"))
        self.g, self.m0 = mv(self.x["g"], torch.float32), mv(self.x["m0"], torch.float32)
        self.kind, self.C, self.backward, self.layout, self.saved = cfg["kind"], cfg["chunk"], cfg["backward"], layout, saved
        B, H, T, dk, dv = (cfg[n] for n in ("B", "H", "T", "dk", "dv"))
        self.tokens, self.th = B * T, B * H * T
        el = 1 if cfg["dtype"] == "bf16" else 0
        self.p = pkg.make_params(B, H, T, dk, dv, self.C, self.kind, el, flags=pkg.FLAG_SAVE_STATES if saved else 0)
        p_other = pkg.make_params(B, H, T, dk, dv, self.C, self.kind, el, flags=0 if saved else pkg.FLAG_SAVE_STATES)
        need = max(pkg.lsm_chunk_fwd_workspace_bytes(pp) for pp in (self.p, p_other))
        need = max(need, max(pkg.lsm_chunk_bwd_workspace_bytes(pp) for pp in (self.p, p_other)), 256)
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        if layout == 1:   # the same values, token-major
            self.q, self.k, self.v, self.d_o = (t_.transpose(1, 2).contiguous() for t_ in (self.q, self.k, self.v, self.d_o))
            if self.kind in (wl.KIND_SCALAR, wl.KIND_VECTOR):
                self.g = self.g.transpose(1, 2).contiguous()

    def step(self, saved=None):
        pkg = self.pkg
        saved = self.saved if saved is None else saved
        out = pkg.lsm_chunk_fwd(self.q, self.k, self.v, self.g, self.kind, self.C, self.m0, workspace=self.ws,
                                layout=self.layout, save_states=saved)
        grads = pkg.lsm_chunk_bwd(self.q, self.k, self.v, self.g, self.kind, self.d_o, self.C, self.m0, workspace=self.ws,
                                  layout=self.layout, states_saved=saved) if self.backward else None
        return out, grads

    def settle(self, seconds=0.25, **kw):
        """Untimed steps until the clocks have settled under this load (a fresh process starts at idle clocks and
        the first steps read about 10 % slow); not part of the warm-up count."""
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(5):
                self.step(**kw)
            self.torch.cuda.synchronize()

    def timed(self, steps, warmup, **kw):
        self.settle(**kw)
        for _ in range(warmup):
            self.step(**kw)
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            last = self.step(**kw)
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps, last

    def parity(self, last, pairs):
        """Every output element of the sampled (b,h) pairs against the fp64 oracle: raw max|x-ref|/RMS(ref), and
        with the half-ulp of the bf16 output container discounted (for the four bf16-stored tensors)."""
        import numpy as np
        from oracle import lsm_oracle_bwd, lsm_oracle_fwd
        x, wl, kind = self.x, self.wl, self.kind
        ib, ih = [p_[0] for p_ in pairs], [p_[1] for p_ in pairs]
        take = lambda a: None if a is None else np.ascontiguousarray(a[ib, ih][None])
        gs = None if x["g"] is None else (np.ascontiguousarray(x["g"][ih]) if kind == wl.KIND_HEAD else take(x["g"]))
        c0 = time.perf_counter()
        o_ref, mT_ref = lsm_oracle_fwd(take(x["q"]), take(x["k"]), take(x["v"]), gs, kind, take(x["m0"]))
        r_ref = lsm_oracle_bwd(take(x["q"]), take(x["k"]), take(x["v"]), gs, kind, take(x["d_o"]), take(x["m0"])) if self.backward else None
        sec = time.perf_counter() - c0
        (o, mT), grads = last
        if self.layout == 1:   # back to the order of the oracle's arrays
            o = o.transpose(1, 2)
            if grads:
                grads = {n_: (t_.transpose(1, 2) if (t_ is not None and t_.dim() >= 3 and n_ != "d_init_state") else t_)
                         for n_, t_ in grads.items()}
        pick = lambda t_: t_[ib, ih].float().cpu().numpy().astype(np.float64)[None]
        ulp = BF16_HALF_ULP if self.cfg["dtype"] == "bf16" else 0.0
        rep, raw = {}, {}
        def put(name, got, ref, u):
            rep[name] = rel_err(got, ref, u)
            if u:
                raw[name] = rel_err(got, ref, 0.0)
        put("o", pick(o), o_ref, ulp)
        put("final_state", pick(mT), mT_ref, 0.0)
        if self.backward:
            for n_ in ("dq", "dk", "dv"):
                put(n_, pick(grads[n_]), r_ref[n_], ulp)
            put("d_init_state", pick(grads["d_init_state"]), r_ref["d_m0"], 0.0)
            if kind in (wl.KIND_SCALAR, wl.KIND_VECTOR):
                put("dg", pick(grads["dg"]), r_ref["dg"], 0.0)
        return rep, raw, sec, len(pairs) * self.cfg["T"]


def sample_pairs(cfg, n=2):
    B, H = cfg["B"], cfg["H"]
    return [(0, 0), (B - 1, H - 1)][:n] if B * H > 1 else [(0, 0)]


def summarise(w, sec):
    cfg = w.cfg
    ffl, bfl = algorithmic_flops_per_token_head(cfg)
    tflops = (ffl + (bfl if w.backward else 0)) * w.th / sec / 1e12
    ab = algorithmic_bytes_per_token_head(cfg, "both" if w.backward else "fwd") * w.th
    return {"ms_per_step": sec * 1e3, "tokens_per_s": w.tokens / sec, "tflops": tflops,
            "mfma_peak_frac": tflops / MFMA_BF16_PEAK_TFLOPS, "hbm_frac_whole_step": ab / sec / 1e9 / HBM_PEAK_GBS,
            "algorithmic_bytes_per_step": ab}


def calibrate(pkg, torch, dev):
    """Achievable peaks of this GPU, measured now: a streaming copy (1 GiB, read + write) and a loop of nothing but
    bf16 MFMAs, both with the library's own calibration kernels."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    out = torch.empty(2048 * 256, dtype=torch.float32, device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for _ in range(3):
        pkg.lsm_calib_copy(dst, src)
        flops = pkg.lsm_calib_mfma(out, 2048, 2048)
    torch.cuda.synchronize()
    reps = 5
    ev[0].record()
    for _ in range(reps):
        pkg.lsm_calib_copy(dst, src)
    ev[1].record()
    ev[2].record()
    for _ in range(reps):
        pkg.lsm_calib_mfma(out, 2048, 2048)
    ev[3].record()
    torch.cuda.synchronize()
    copy_gbs = 2 * src.numel() * reps / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
    mfma_tf = flops * reps / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e12
    del src, dst, out
    return {"copy_GBps_read_plus_write": copy_gbs, "copy_bytes": 1 << 30, "mfma_bf16_TFLOPs": mfma_tf,
            "what": "lsm_calib_copy on 1 GiB (bytes read + written over time) and lsm_calib_mfma (2048 workgroups x 4 waves x "
                    "8192 independent 32x32x16 bf16 MFMAs on register operands), same process, same clocks"}


def delta_bench(steps, warmup, check):
    """Forward and backward of the delta-rule rows (DeltaNet, Gated DeltaNet): 256 sequences of 2048 tokens, the shape of
    a training batch at the paper's 2K context (one workgroup walks a sequence, so 256 sequences fill the chip), and
    the metric's own shape (64 sequences of 8192 tokens) for what few sequences cost.  Per row: host-clock time per
    forward and per forward + backward step, HIP-event kernel averages, compulsory bytes over time, and sampled (b,h)
    pairs against the fp64 oracle and its adjoint."""
    import ctypes
    import numpy as np
    import torch
    import lsm_workloads as wl
    import paper_2503_05447_amd as pkg
    dev = torch.device("cuda:0")
    out = {"what": "lsm_delta_fwd / lsm_delta_bwd, bf16, d_k = d_v = 128, chunk 64; keys of unit length, b = sigmoid(N(0,1)), "
                   "DeltaNet a = b, Gated DeltaNet log a = -softplus(N(0,1) + 3); d_o ~ N(0,1)"}
    for (B, H, T) in ((16, 16, 2048), (4, 16, 8192)):
        for gated in (False, True):
            x = wl.make_delta_inputs(B, H, T, 128, 128, gated, seed=wl.BASE_SEED + 20 + int(gated) + T)
            mv = lambda a, dt: None if a is None else torch.from_numpy(a).to(dev).to(dt).contiguous()
            q, k, v, d_o = (mv(x[n_], torch.bfloat16) for n_ in ("q", "k", "v", "d_o"))
            la, be, bw = (mv(x[n_], torch.float32) for n_ in ("log_alpha", "beta", "b"))
            p = pkg.make_params(B, H, T, 128, 128, 64, pkg.DECAY_SCALAR if gated else pkg.DECAY_NONE, 1)
            ws = torch.empty(pkg.library().lsm_delta_fwd_workspace_bytes(ctypes.byref(p)), dtype=torch.uint8, device=dev)
            wsb = torch.empty(pkg.library().lsm_delta_bwd_workspace_bytes(ctypes.byref(p)), dtype=torch.uint8, device=dev)
            step = lambda: pkg.lsm_delta_fwd(q, k, v, la, be, bw, workspace=ws)
            bstep = lambda: pkg.lsm_delta_bwd(q, k, v, d_o, la, be, bw, workspace=wsb)
            # the pair as a training step runs it: the forward call keeps what the backward call needs of it
            fkeep = lambda: pkg.lsm_delta_fwd(q, k, v, la, be, bw, workspace=wsb, save_states=True)
            bkeep = lambda: pkg.lsm_delta_bwd(q, k, v, d_o, la, be, bw, workspace=wsb, states_saved=True)
            t0 = time.perf_counter()
            while time.perf_counter() - t0 < 0.25:   # settle the clocks, as for the headline
                for _ in range(5):
                    step()
                torch.cuda.synchronize()
            for _ in range(warmup):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                o, mT = step()
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t0) / steps
            for _ in range(min(warmup, 3)):
                step()
                grads = bstep()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
                grads = bstep()
            torch.cuda.synchronize()
            sec_fb_re = (time.perf_counter() - t0) / steps
            for _ in range(min(warmup, 3)):
                fkeep()
                grads = bkeep()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fkeep()
                grads = bkeep()
            torch.cuda.synchronize()
            sec_fb = (time.perf_counter() - t0) / steps
            pkg.lsm_profile_start()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            per = {}
            for name, ms in pkg.lsm_profile_stop():
                per.setdefault(name, []).append(ms)
            pkg.lsm_profile_start()
            for _ in range(steps):
                fkeep()
                bkeep()
            torch.cuda.synchronize()
            perb = {}
            for name, ms in pkg.lsm_profile_stop():
                perb.setdefault(name, []).append(ms)
            th = B * H * T
            ab = th * (4 * 256 + 4 * 2)   # q, k, v, o in bf16; two per-token parameters
            abb = th * (7 * 256 + 4 * 4)  # backward: q, k, v, d_o read, dq, dk, dv written; parameters and their gradients
            # chunk-dense flops per token-head: scores, A U, Q S, state update (as the diagonal kinds) + K K^T,
            # T [V | K], What S
            fl = th * (2 * 64 * 256 + 2 * 2 * 128 * 128 + 2 * 64 * 128 + 2 * 64 * 256 + 2 * 128 * 128)
            e = {"B": B, "H": H, "T": T, "ms_per_step": sec * 1e3, "tokens_per_s": B * T / sec, "steps": steps,
                 "kernel_ms": {n_: float(np.mean(v_)) for n_, v_ in per.items()},
                 "ms_per_step_fwd_bwd": sec_fb * 1e3, "tokens_per_s_fwd_bwd": B * T / sec_fb,
                 "fwd_bwd_states": "kept by the forward call", "ms_per_step_fwd_bwd_recomputing": sec_fb_re * 1e3,
                 "kernel_ms_fwd_bwd": {n_: float(np.sum(v_)) / steps for n_, v_ in perb.items()},
                 "algorithmic_bytes_per_step_fwd_bwd": ab + abb,
                 "hbm_frac_whole_step_fwd_bwd": (ab + abb) / sec_fb / 1e9 / HBM_PEAK_GBS,
                 "algorithmic_bytes_per_step": ab, "hbm_frac_whole_step": ab / sec / 1e9 / HBM_PEAK_GBS,
                 "tflops_chunk_dense": fl / sec / 1e12, "mfma_peak_frac": fl / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS}
            if check:
                from oracle import delta_oracle_bwd, delta_oracle_fwd
                pairs = [(0, 0), (B - 1, H - 1)]
                ib, ih = [p_[0] for p_ in pairs], [p_[1] for p_ in pairs]
                take = lambda a: None if a is None else np.ascontiguousarray(a[ib, ih][None])
                c0 = time.perf_counter()
                o_ref, mT_ref = delta_oracle_fwd(take(x["q"]), take(x["k"]), take(x["v"]), take(x["log_alpha"]), take(x["beta"]),
                                                 take(x["b"]), None)
                osec = time.perf_counter() - c0
                pick = lambda t_: t_[ib, ih].float().cpu().numpy().astype(np.float64)[None]
                e["parity_err_over_rms"] = {"o": rel_err(pick(o), o_ref, BF16_HALF_ULP), "final_state": rel_err(pick(mT), mT_ref, 0.0)}
                e["parity_err_over_rms_raw"] = {"o": rel_err(pick(o), o_ref, 0.0)}
                e["parity_pairs"] = pairs
                e["cpu_oracle_tokens_per_s"] = len(pairs) * T / osec
                r_ref = delta_oracle_bwd(take(x["q"]), take(x["k"]), take(x["v"]), take(x["d_o"]), take(x["log_alpha"]),
                                         take(x["beta"]), take(x["b"]))
                names = dict(dq="dq", dk="dk", dv="dv", d_log_alpha="d_log_alpha", d_beta="d_beta", d_b="d_b", d_init_state="d_m0")
                for n_, rn in names.items():
                    if grads[n_] is None:
                        continue
                    stored = n_ in ("dq", "dk", "dv")
                    e["parity_err_over_rms"][n_] = rel_err(pick(grads[n_]), r_ref[rn], BF16_HALF_ULP if stored else 0.0)
                    if stored:
                        e["parity_err_over_rms_raw"][n_] = rel_err(pick(grads[n_]), r_ref[rn], 0.0)
            out["%s_B%d_T%d" % ("gated_deltanet" if gated else "deltanet", B, T)] = e
            del q, k, v, d_o, la, be, bw, ws, wsb, o, mT, grads
            torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration 1..5 of the headline line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--layout", type=int, default=0, choices=(0, 1),
                    help="0: [B,H,T,d] as BASELINE.json's configurations are written; 1: the same data token-major [B,T,H,d]")
    ap.add_argument("--states", choices=("recompute", "saved"), default="saved",
                    help="states of the backward pass: kept by the forward call in the shared workspace, or computed again "
                         "from the inputs; the other mode is timed too and reported beside the headline")
    ap.add_argument("--no-microbench", action="store_true",
                    help="skip the LDS-resident intra-chunk micro-benchmark, the decode step and the calibration kernels "
                         "(profiling runs: they launch other kernels)")
    ap.add_argument("--no-all-configs", action="store_true", help="skip the other four configurations")
    ap.add_argument("--no-delta", action="store_true", help="skip the delta-rule rows (lsm_delta_fwd)")
    ap.add_argument("--delta-only", action="store_true", help="run only the delta-rule rows and print their block (profiling runs)")
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
    if args.delta_only:
        print(json.dumps({"delta_rule": delta_bench(max(5, min(args.steps, 50)), min(args.warmup, 10), not args.no_check)}))
        return
    saved = args.states == "saved"
    w = Workload(args.config, args.layout, saved)
    cfg, kind, C = w.cfg, w.kind, w.C
    B, H, T, dk, dv = (cfg[n] for n in ("B", "H", "T", "dk", "dv"))
    kept = {True: "saved by the forward call", False: "recomputed"}

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    sec, last = w.timed(args.steps, args.warmup)
    # Per-kernel durations: the same K steps once more with a pair of HIP events around every launch, on
    # the launch stream.  The events keep consecutive kernels from overlapping and cost several percent of
    # a step, so this pass is timed on its own (ms_per_step_with_events) and not reported as the throughput.
    pkg.lsm_profile_start()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        w.step()
    torch.cuda.synchronize()
    sec_events = (time.perf_counter() - t2) / args.steps
    prof = pkg.lsm_profile_stop()

    per_kernel = {}
    for name, ms in prof:
        per_kernel.setdefault(name, []).append(ms)
    launches = {n: len(v_) / args.steps for n, v_ in per_kernel.items()}
    kavg = {n: float(np.mean(v_)) for n, v_ in per_kernel.items()}
    # roofline of the dominant kernel among those that move the method's own inputs and outputs
    cand = {n: t_ for n, t_ in kavg.items() if KERNEL_PASS.get(n)}
    dominant = max(cand, key=cand.get)
    abytes = algorithmic_bytes_per_token_head(cfg, KERNEL_PASS[dominant]) * w.th
    achieved = abytes / (kavg[dominant] * 1e-3) / 1e9
    # pass level: the compulsory bytes of a pass over the summed durations of all its kernels
    tot_ms = sum(kavg[n] * launches[n] for n in kavg)
    passes = {"whole_step": {"algorithmic_GBps": algorithmic_bytes_per_token_head(cfg, "both" if w.backward else "fwd") * w.th / (tot_ms * 1e-3) / 1e9,
                             "kernel_ms_sum": tot_ms}}
    passes["whole_step"]["frac_of_hbm_peak"] = passes["whole_step"]["algorithmic_GBps"] / HBM_PEAK_GBS

    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            key = cfg["name"] + ("" if pkg.keeps_states(w.p) == 1 else "_recompute")
            traffic = json.load(f).get(key, {}).get(dominant)
    except (OSError, ValueError):
        pass

    s = summarise(w, sec)
    ffx, bfx = algorithmic_flops_per_token_head(cfg, causal_exact=True)
    result = {
        "metric": "LSM chunkwise fwd+bwd tokens/s and TFLOP/s (%MFMA peak) at H=16,d=128,T=8192",
        "value": s["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": s["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": cfg["name"], "B": B, "H": H, "T": T, "d_k": dk, "d_v": dv, "chunk": C,
                   "decay_kind": wl.KIND_NAMES[kind], "passes": "fwd+bwd" if w.backward else "fwd",
                   "kernel_path": "mfma" if pkg.kernel_path(w.p) == 1 else "generic",
                   "layout": "BTHD" if args.layout else "BHTD", "bwd_states": kept[pkg.keeps_states(w.p) == 1]},
        "tflops": s["tflops"], "mfma_peak_frac": s["mfma_peak_frac"],
        "tflops_causal_exact": (ffx + (bfx if w.backward else 0)) * w.th / sec / 1e12,
        "flop_convention": "tflops: chunk-dense (every C x C block counted in full, as Algorithm 2 computes it); "
                           "tflops_causal_exact: only pairs r <= j",
        "hbm_frac_whole_step": s["hbm_frac_whole_step"],
        "kernel_ms": kavg, "kernel_launches_per_step": launches, "ms_per_step_with_events": sec_events * 1e3,
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE of a committed run, not this run)",
                     "algorithmic_bytes_per_launch": abytes,
                     "kernels_without_algorithmic_output": sorted(n for n in kavg if not KERNEL_PASS.get(n)),
                     "passes": passes},
    }

    if w.backward and not args.no_microbench:   # the same steps with the other treatment of the states
        sec2, _ = w.timed(args.steps, args.warmup, saved=not saved)
        p_keep = pkg.make_params(B, H, T, dk, dv, C, kind, 1 if cfg["dtype"] == "bf16" else 0, flags=pkg.FLAG_SAVE_STATES)
        other = kept[False] if saved else kept[pkg.keeps_states(p_keep) == 1]
        result["other_bwd_states"] = {"bwd_states": other, "ms_per_step": sec2 * 1e3, "value": w.tokens / sec2,
                                      "unit": "tokens/s"}

    if not args.no_microbench:
        cal = calibrate(pkg, torch, dev)
        result["calibration"] = cal
        result["roofline"]["frac_of_calibrated_copy"] = achieved / cal["copy_GBps_read_plus_write"]
        result["mfma_frac_of_calibrated_peak"] = s["tflops"] / cal["mfma_bf16_TFLOPs"]

    if pkg.kernel_path(w.p) == 1 and kind != wl.KIND_VECTOR and not args.no_microbench and args.layout == 0:
        # Intra-chunk phase apart from HBM: the per-chunk output kernel with its compute phase repeated on
        # LDS-resident tiles; the time of one pass is the slope between two repeat counts.
        R = 33
        o_mb = torch.empty_like(last[0][0])
        o_plain, _ = pkg.lsm_chunk_fwd(w.q, w.k, w.v, w.g, kind, C, None, workspace=w.ws)
        ws_mb = pkg.lsm_bench_intra_chunk_workspace(w.q, w.k, w.v, w.g, kind, C)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        pkg.lsm_bench_intra_chunk(w.q, w.k, w.v, w.g, kind, o_mb, ws_mb, 1, C)
        pkg.lsm_profile_start()
        pkg.lsm_bench_intra_chunk(w.q, w.k, w.v, w.g, kind, o_mb, ws_mb, 1, C)
        pkg.lsm_bench_intra_chunk(w.q, w.k, w.v, w.g, kind, o_mb, ws_mb, R, C)
        mb = [ms for name, ms in pkg.lsm_profile_stop() if name == "mfma_output"]
        t1_ms, tR_ms = mb[0], mb[1]
        pass_s = (tR_ms - t1_ms) / (R - 1) * 1e-3
        chunks = B * H * ((T + C - 1) // C)
        alg = chunks * (2 * C * C * (dk + dv) + 2 * C * dk * dv)          # dense C x C block + Q S_c (Algorithm 2)
        # issued MFMA 32x32x16 per chunk: Q S_c 4 x 16, three score blocks x 8, A V with head + remainder 4 x 12
        issued = chunks * 136 * 2 * 32 * 32 * 16
        mbres = {
            "what": "per-chunk forward kernel (scores, mask/decay, A V, Q S_c) on materialised chunk states, compute phase "
                    "repeated on LDS-resident tiles (benchmark aid; the product path fuses this phase into the chunk walker)",
            "repeats": R, "ms_one_pass": pass_s * 1e3, "ms_streamed_kernel": t1_ms,
            "algorithmic_tflops": alg / pass_s / 1e12, "algorithmic_frac_of_mfma_peak": alg / pass_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "algorithmic_frac_of_calibrated_mfma_peak": alg / pass_s / 1e12 / result["calibration"]["mfma_bf16_TFLOPs"],
            "issued_mfma_tflops": issued / pass_s / 1e12, "issued_frac_of_mfma_peak": issued / pass_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "max_abs_diff_to_forward": float((o_mb.float() - o_plain.float()).abs().max())}
        try:   # the matrix-pipe utilisation the hardware counters give for the same launches (collected under rocprofv3)
            with open(os.path.join(ROOT, "profiles", "mfma_counters.json")) as f:
                mbres["rocprof_counters"] = json.load(f).get(cfg["name"] + "_intra_chunk_microbench")
        except (OSError, ValueError):
            pass
        result["intra_chunk_microbench"] = mbres
        del ws_mb, o_mb, o_plain

    if not args.no_microbench:
        # Recurrent decoding step (lsm_step) on the heads of this workload: state read + written once per step.
        tdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        dec = {}
        for Bd in (16, 256):
            qd = torch.randn(Bd, H, dk, device=dev).to(tdt)
            kd = torch.randn(Bd, H, dk, device=dev).to(tdt) / dk ** 0.5
            vd = torch.randn(Bd, H, dv, device=dev).to(tdt)
            gd = {wl.KIND_NONE: None, wl.KIND_HEAD: w.g}.get(kind, None)
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
        x = w.x
        # bounded sample: the first `nb` batch elements of the same workload (all heads, full T)
        nb = max(1, min(B, (1 << 20) // (H * T) or 1))
        sl = slice(0, nb)
        gs = x["g"] if (x["g"] is None or kind == wl.KIND_HEAD) else x["g"][sl]
        m0s = None if x["m0"] is None else x["m0"][sl]
        c0 = time.perf_counter()
        o_ref, mT_ref = lsm_oracle_fwd(x["q"][sl], x["k"][sl], x["v"][sl], gs, kind, m0s)
        r_ref = lsm_oracle_bwd(x["q"][sl], x["k"][sl], x["v"][sl], gs, kind, x["d_o"][sl], m0s) if w.backward else None
        c1 = time.perf_counter()
        result["cpu_baseline"] = {"value": nb * T / (c1 - c0), "unit": "tokens/s", "cores": oracle_threads(),
                                  "kind": "oracle",
                                  "sample": "batch elements 0..%d of the same workload, all %d heads, full T=%d, %s"
                                            % (nb - 1, H, T, "fwd+bwd" if w.backward else "fwd"),
                                  "seconds": c1 - c0}
        if not args.no_check:
            (o, mT), grads = last
            if args.layout == 1:   # back to the order of the oracle's arrays
                o = o.transpose(1, 2)
                if grads:
                    grads = {n_: (t_.transpose(1, 2) if (t_ is not None and t_.dim() >= 3 and n_ != "d_init_state") else t_)
                             for n_, t_ in grads.items()}
            host = lambda t_: t_.float().cpu().numpy().astype(np.float64)
            ulp = BF16_HALF_ULP if cfg["dtype"] == "bf16" else 0.0   # half-ulp of the bf16 output container
            par = {"o": rel_err(host(o[sl]), o_ref, ulp), "final_state": rel_err(host(mT[sl]), mT_ref, 0.0)}
            raw = {"o": rel_err(host(o[sl]), o_ref, 0.0)}
            if w.backward:
                for n_ in ("dq", "dk", "dv"):
                    par[n_] = rel_err(host(grads[n_][sl]), r_ref[n_], ulp)
                    raw[n_] = rel_err(host(grads[n_][sl]), r_ref[n_], 0.0)
                if kind in (wl.KIND_SCALAR, wl.KIND_VECTOR):
                    par["dg"] = rel_err(host(grads["dg"][sl]), r_ref["dg"], 0.0)
            result["parity_err_over_rms"] = par
            # the same maxima without the discount of the bf16 output container's own half-ulp (fp32-stored tensors
            # are never discounted); a bf16 container alone costs up to 2^-8 |x| / RMS at the largest elements
            result["parity_err_over_rms_raw"] = raw if ulp else {}
            result["parity_tolerance"] = {"f32": 1e-4, "bf16": 2e-2}[cfg["dtype"]]

    if not args.no_delta and not args.no_microbench:
        del w
        torch.cuda.empty_cache()
        result["delta_rule"] = delta_bench(max(5, min(args.steps, 50)), min(args.warmup, 10), not args.no_check)
        w = None

    if not args.no_all_configs:
        # The other configurations, each on its full shape: a shorter timed run, and every output element of two
        # (b,h) pairs against the oracle.
        del last
        s = {n_: v_ for n_, v_ in s.items()}
        allc = {}
        for idx in range(1, 6):
            if idx == args.config:
                allc[cfg["name"]] = {**s, "steps": args.steps, "see": "headline fields of this line"}
                continue
            del w
            torch.cuda.empty_cache()
            w = Workload(idx, 0, saved)
            n_steps = max(5, min(args.steps, 20))
            sec_i, last_i = w.timed(n_steps, min(args.warmup, 5))
            entry = summarise(w, sec_i)
            entry["steps"] = n_steps
            entry["kernel_path"] = "mfma" if pkg.kernel_path(w.p) == 1 else "generic"
            if not args.no_check:
                rep, raw, osec, otok = w.parity(last_i, sample_pairs(w.cfg))
                entry["parity_err_over_rms"] = rep
                entry["parity_err_over_rms_raw"] = raw
                entry["parity_pairs"] = sample_pairs(w.cfg)
            allc[w.cfg["name"]] = entry
            del last_i
        result["all_configs"] = allc
    print(json.dumps(result))


if __name__ == "__main__":
    main()
