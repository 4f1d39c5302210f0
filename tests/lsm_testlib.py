"""Helpers of the GPU parity tests: move seeded inputs to the device, call the C-ABI
binding, run the fp64 oracle on the same values, and compare tensor by tensor."""
import numpy as np

import lsm_workloads as wl

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max |x - ref| / RMS(ref), per tensor


def to_device(x):
    import torch
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if x["dtype"] == "bf16" else torch.float32
    def mv(a, dt):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt).contiguous()
    t = {n: mv(x[n], tdt) for n in ("q", "k", "v", "d_o")}
    t.update({n: mv(x[n], torch.float32) for n in ("g", "m0", "d_mT")})
    return t


def gpu_forward(x, chunk, t=None, want_final=True):
    import paper_2503_05447_amd as pkg
    t = t or to_device(x)
    return pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], x["kind"], chunk, t["m0"], want_final_state=want_final)


def gpu_backward(x, chunk, t=None, **kw):
    import paper_2503_05447_amd as pkg
    t = t or to_device(x)
    return pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], x["kind"], t["d_o"], chunk, t["m0"], t["d_mT"], **kw)


def host(t):
    return None if t is None else t.detach().float().cpu().numpy().astype(np.float64)


BF16_STORED = ("o", "dq", "dk", "dv")   # tensors the library returns in the element type of q
BF16_HALF_ULP = 2.0 ** -8               # half an ulp of a bf16 number, relative to its magnitude (upper bound)


def rel_err(got, ref, storage_ulp=0.0):
    """max (|got-ref| - storage_ulp*|ref|)_+ / RMS(ref); absolute when RMS(ref) == 0.

    storage_ulp > 0 discounts the one rounding of an fp32 result into a bf16 output container
    (at most half an ulp of the stored value), so that only rounding INSIDE the path is measured,
    as it is on the input side where the oracle consumes the already-rounded bf16 inputs."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values in GPU result"
    if not ref.size:
        return 0.0
    rms = float(np.sqrt(np.mean(ref ** 2)))
    e = float(np.maximum(np.abs(got - ref) - storage_ulp * np.abs(ref), 0.0).max())
    return e / rms if rms > 0 else e


def elementwise_rel_err(got, ref):
    """max relative error over elements with |ref| >= RMS(ref)."""
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref ** 2))
    m = np.abs(ref) >= rms
    if rms == 0 or not m.any():
        return 0.0
    return float((np.abs(np.asarray(got, dtype=np.float64) - ref)[m] / np.abs(ref)[m]).max())


def check(name, got, ref, dtype, report=None):
    ulp = BF16_HALF_ULP if (dtype == "bf16" and name in BF16_STORED) else 0.0
    err = rel_err(got, ref, ulp)
    if report is not None:
        report[name] = err
        if ulp:
            report[name + "_raw"] = rel_err(got, ref)
    assert err <= TOL[dtype], "%s: err/rms %.3e > %.1e" % (name, err, TOL[dtype])
    if dtype == "f32":
        e2 = elementwise_rel_err(got, ref)
        assert e2 <= TOL[dtype], "%s: elementwise rel err %.3e" % (name, e2)
    return err


def oracle_all(x, backward=True):
    from oracle import lsm_oracle_bwd, lsm_oracle_fwd
    o, mT = lsm_oracle_fwd(x["q"], x["k"], x["v"], x["g"], x["kind"], x["m0"])
    r = lsm_oracle_bwd(x["q"], x["k"], x["v"], x["g"], x["kind"], x["d_o"], x["m0"], x["d_mT"]) if backward else None
    return o, mT, r


def compare_case(x, chunk, backward=True):
    """Full element-by-element comparison of one seeded case; returns the error report."""
    import torch
    t = to_device(x)
    o, mT = gpu_forward(x, chunk, t)
    r = gpu_backward(x, chunk, t) if backward else None
    torch.cuda.synchronize()
    o_ref, mT_ref, r_ref = oracle_all(x, backward)
    rep = {}
    check("o", host(o), o_ref, x["dtype"], rep)
    check("final_state", host(mT), mT_ref, x["dtype"], rep)
    if backward:
        check("dq", host(r["dq"]), r_ref["dq"], x["dtype"], rep)
        check("dk", host(r["dk"]), r_ref["dk"], x["dtype"], rep)
        check("dv", host(r["dv"]), r_ref["dv"], x["dtype"], rep)
        check("d_init_state", host(r["d_init_state"]), r_ref["d_m0"], x["dtype"], rep)
        if x["kind"] != wl.KIND_NONE:
            check("dg", host(r["dg"]), r_ref["dg"], x["dtype"], rep)
        else:
            assert r["dg"] is None
    return rep


def select_heads(x, pairs):
    """Restrict a case to the given (b,h) pairs, as a B=1, H=len(pairs) case (heads are independent).
    For the per-head kind all pairs must share nothing: g is gathered per pair."""
    idx_b = [p[0] for p in pairs]
    idx_h = [p[1] for p in pairs]
    def take(a):
        return None if a is None else np.ascontiguousarray(a[idx_b, idx_h][None])
    y = dict(x)
    for n in ("q", "k", "v", "d_o", "m0", "d_mT"):
        y[n] = take(x[n])
    if x["kind"] == wl.KIND_HEAD:
        y["g"] = np.ascontiguousarray(x["g"][idx_h])
    elif x["g"] is not None:
        y["g"] = take(x["g"])
    y["B"], y["H"] = 1, len(pairs)
    return y
