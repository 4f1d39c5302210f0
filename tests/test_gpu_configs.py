"""The five benchmark configurations at FULL size, in the launch configuration bench.py times:
the GPU runs the whole workload, the fp64 oracle recomputes a sample of (b,h) pairs (sequences of
different pairs are independent, so a pair can be recomputed alone) and every output element of
those pairs is compared.  Same tolerances as the small parity tests."""
import numpy as np
import pytest

import lsm_workloads as wl
from lsm_testlib import check, gpu_backward, gpu_forward, host, oracle_all, select_heads, to_device

pytestmark = pytest.mark.gpu


def run_config(index, pairs, keep=False):
    """keep: bench.py's default, the forward call leaves its chunk states for the backward call."""
    import torch
    import paper_2503_05447_amd as pkg
    x, cfg = wl.make_config(index)
    t = to_device(x)
    if keep:
        ws = pkg.lsm_chunk_workspace(t["q"], t["k"], t["v"], t["g"], cfg["kind"], cfg["chunk"], save_states=True)
        o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], cfg["kind"], cfg["chunk"], t["m0"], workspace=ws,
                                  save_states=True)
        r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], cfg["kind"], t["d_o"], cfg["chunk"], t["m0"], t["d_mT"],
                              workspace=ws, states_saved=True)
    else:
        o, mT = gpu_forward(x, cfg["chunk"], t)
        r = gpu_backward(x, cfg["chunk"], t) if cfg["backward"] else None
    torch.cuda.synchronize()
    y = select_heads(x, pairs)
    o_ref, mT_ref, r_ref = oracle_all(y, cfg["backward"])
    ib, ih = [p[0] for p in pairs], [p[1] for p in pairs]
    pick = lambda a: host(a[ib, ih][None])
    rep = {}
    dt = cfg["dtype"]
    check("o", pick(o), o_ref, dt, rep)
    check("final_state", pick(mT), mT_ref, dt, rep)
    if cfg["backward"]:
        for key in ("dq", "dk", "dv"):
            check(key, pick(r[key]), r_ref[key], dt, rep)
        check("d_init_state", pick(r["d_init_state"]), r_ref["d_m0"], dt, rep)
        if cfg["kind"] in (wl.KIND_SCALAR, wl.KIND_VECTOR):
            check("dg", pick(r["dg"]), r_ref["dg"], dt, rep)
    p = pkg.make_params(cfg["B"], cfg["H"], cfg["T"], cfg["dk"], cfg["dv"], cfg["chunk"], cfg["kind"],
                        1 if dt == "bf16" else 0)
    print(cfg["name"], "path", pkg.kernel_path(p), rep)
    return x, cfg, r, r_ref, rep


def test_config1_basic_linear_attention_fp32_full():
    run_config(0, [(0, 0), (0, 1)])


@pytest.mark.parametrize("keep", [False, True])
def test_config2_fixed_per_head_decay(keep):
    # the per-head decay gradient sums over batch and time: take every batch element of two heads
    for h in (0, 15):
        pairs = [(b, h) for b in range(8)]
        x, cfg, r, r_ref, _ = run_config(1, pairs, keep)
        got = host(r["dg"])[h]
        ref = r_ref["dg"].sum()           # the oracle saw the 8 pairs as 8 heads sharing g_h
        scale = np.sqrt(np.mean(r_ref["dg"] ** 2)) * np.sqrt(len(pairs))
        assert abs(got - ref) <= 2e-2 * max(scale, abs(ref)), (h, got, ref)


@pytest.mark.parametrize("keep", [False, True])
def test_config3_scalar_decay_metric_shape(keep):
    import paper_2503_05447_amd as pkg
    x, cfg, *_ = run_config(2, [(0, 0), (1, 7), (3, 15)], keep)
    p = pkg.make_params(cfg["B"], cfg["H"], cfg["T"], cfg["dk"], cfg["dv"], cfg["chunk"], cfg["kind"], 1,
                        flags=pkg.FLAG_SAVE_STATES if keep else 0)
    assert pkg.kernel_path(p) == 1, "the metric shape must run on the MFMA kernels"
    assert pkg.keeps_states(p) == (1 if keep else 0)


@pytest.mark.parametrize("keep", [False, True])
def test_config4_vector_decay(keep):
    run_config(3, [(0, 3), (3, 12)], keep)


def test_config5_long_sequence_with_carried_state():
    run_config(4, [(0, 0), (0, 31)])


def _equal(a, b):
    import torch
    if a is None or b is None:
        return a is None and b is None
    return torch.equal(a, b)


@pytest.mark.parametrize("index", [1, 2, 4])
def test_repeated_calls_at_full_size_are_bitwise_identical(index):
    """The walkers split a workgroup into groups of waves that hand tiles to each other through LDS between barriers.
    Every reduction order is fixed, so a call repeated on the same inputs must reproduce every output bit for bit;
    a hand-over that was not ordered by a barrier would show as a difference on a chip that is busy throughout."""
    import torch
    import paper_2503_05447_amd as pkg
    x, cfg = wl.make_config(index)
    t = to_device(x)
    def once():
        o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], cfg["kind"], cfg["chunk"], t["m0"])
        r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], cfg["kind"], t["d_o"], cfg["chunk"], t["m0"], t["d_mT"])
        torch.cuda.synchronize()
        return dict(o=o, mT=mT, **{k: r[k] for k in ("dq", "dk", "dv", "dg", "d_init_state")})
    first = once()
    for rep in range(4):
        again = once()
        for name, val in first.items():
            assert _equal(val, again[name]), (cfg["name"], name, rep)


@pytest.mark.parametrize("gated", [False, True])
@pytest.mark.parametrize("shape", [(16, 16, 2048), (4, 16, 8192)])
def test_repeated_delta_rule_calls_at_full_size_are_bitwise_identical(shape, gated):
    import torch
    import paper_2503_05447_amd as pkg
    B, H, T = shape
    x = wl.make_delta_inputs(B, H, T, 128, 128, gated, seed=77 + int(gated), init_state=True, d_final=True)
    d = torch.device("cuda:0")
    mv = lambda a, dt: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(d).to(dt).contiguous()
    q, k, v, d_o = (mv(x[n], torch.bfloat16) for n in ("q", "k", "v", "d_o"))
    la, be, bw, m0, d_mT = (mv(x[n], torch.float32) for n in ("log_alpha", "beta", "b", "m0", "d_mT"))
    def once():
        o, mT = pkg.lsm_delta_fwd(q, k, v, la, be, bw, m0)
        r = pkg.lsm_delta_bwd(q, k, v, d_o, la, be, bw, m0, d_mT)
        torch.cuda.synchronize()
        return dict(o=o, mT=mT, **{n: r[n] for n in ("dq", "dk", "dv", "d_log_alpha", "d_beta", "d_b", "d_init_state")})
    first = once()
    for rep in range(3):
        again = once()
        for name, val in first.items():
            assert _equal(val, again[name]), (shape, gated, name, rep)
