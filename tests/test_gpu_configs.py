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
