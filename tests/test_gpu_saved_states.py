"""Saved chunk states: the forward call keeps its states in the workspace and the backward call reads
them instead of computing them again.  Outputs and gradients must meet the same bar against the oracle
as those of the recomputing path, and shapes served by kernels that keep nothing must give exactly what
they give without the flag."""
import numpy as np
import pytest

import lsm_workloads as wl
from lsm_testlib import check, host, oracle_all, to_device

pytestmark = pytest.mark.gpu

KINDS = [wl.KIND_NONE, wl.KIND_HEAD, wl.KIND_SCALAR, wl.KIND_VECTOR]


def run_saved(pkg, t, kind, chunk=64, layout=0, cu=None, **bw):
    ws = pkg.lsm_chunk_workspace(t["q"], t["k"], t["v"], t["g"], kind, chunk, layout, cu, save_states="always")
    o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, chunk, t["m0"], workspace=ws, layout=layout,
                              cu_seqlens=cu, save_states="always")
    r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], chunk, t["m0"], t["d_mT"], workspace=ws,
                          layout=layout, cu_seqlens=cu, states_saved="always", **bw)
    return o, mT, r


@pytest.mark.parametrize("decay", ["weak", "default", "harsh"])
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("shape", [(2, 3, 300, 128, 128), (1, 2, 150, 128, 256)])
def test_saved_states_match_oracle(kind, shape, decay):
    import torch
    import paper_2503_05447_amd as pkg
    B, H, T, dk, dv = shape
    # carried-in states with the decays under which they matter; under the harsh law they would leave a few
    # large leading outputs over a vanishing RMS, and the metric would measure the bf16 container alone
    st = decay != "harsh"
    x = wl.make_inputs(B, H, T, dk, dv, kind, dtype="bf16", seed=1200 + 7 * kind + T, decay=decay, init_state=st,
                       d_final=st)
    t = to_device(x)
    o, mT, r = run_saved(pkg, t, kind)
    torch.cuda.synchronize()
    o_ref, mT_ref, r_ref = oracle_all(x)
    check("o", host(o), o_ref, "bf16")
    check("final_state", host(mT), mT_ref, "bf16")
    for key in ("dq", "dk", "dv"):
        check(key, host(r[key]), r_ref[key], "bf16")
    check("d_init_state", host(r["d_init_state"]), r_ref["d_m0"], "bf16")
    if kind != wl.KIND_NONE:
        check("dg", host(r["dg"]), r_ref["dg"], "bf16")


@pytest.mark.parametrize("kind", [wl.KIND_SCALAR, wl.KIND_VECTOR])
def test_saved_states_without_decay_gradient(kind):
    """d_log_decay not asked for: the remainder planes are not read."""
    import torch
    import paper_2503_05447_amd as pkg
    x = wl.make_inputs(1, 2, 200, 128, 128, kind, dtype="bf16", seed=1300 + kind, decay="weak", init_state=True,
                       d_final=True)
    t = to_device(x)
    _, _, r = run_saved(pkg, t, kind, want_d_log_decay=False)
    torch.cuda.synchronize()
    _, _, r_ref = oracle_all(x)
    assert r["dg"] is None
    for key in ("dq", "dk", "dv"):
        check(key, host(r[key]), r_ref[key], "bf16")


@pytest.mark.parametrize("kind", [wl.KIND_HEAD, wl.KIND_VECTOR])
def test_saved_states_packed_token_major(kind):
    """Packed sequences in the token-major layout, saved against recomputed (same bar as against the oracle)."""
    import torch
    import paper_2503_05447_amd as pkg
    lens = [70, 1, 130, 64, 5]
    T, H = sum(lens), 2
    x = wl.make_inputs(1, H, T, 128, 128, kind, dtype="bf16", seed=1400 + kind, decay="weak")
    rng = np.random.default_rng(5)
    x["m0"] = (rng.standard_normal((len(lens), H, 128, 128)) * 0.1).astype(np.float32)
    x["d_mT"] = (rng.standard_normal((len(lens), H, 128, 128)) * 0.1).astype(np.float32)
    t = to_device(x)
    for n in ("q", "k", "v", "d_o"):
        t[n] = t[n].transpose(1, 2).contiguous()
    if kind == wl.KIND_VECTOR:
        t["g"] = t["g"].transpose(1, 2).contiguous()
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(t["q"].device)
    o, mT, r = run_saved(pkg, t, kind, layout=pkg.LAYOUT_BTHD, cu=cu)
    o0, mT0 = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"], layout=pkg.LAYOUT_BTHD, cu_seqlens=cu)
    r0 = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"],
                           layout=pkg.LAYOUT_BTHD, cu_seqlens=cu)
    torch.cuda.synchronize()
    check("o", host(o), host(o0), "bf16")
    check("final_state", host(mT), host(mT0), "bf16")
    for key in ("dq", "dk", "dv", "dg", "d_init_state"):
        check(key, host(r[key]), host(r0[key]), "bf16")


@pytest.mark.parametrize("kind", KINDS)
def test_flag_is_inert_where_nothing_is_kept(kind):
    """fp32 inputs run on kernels that keep nothing: with the flag they return the very same bits."""
    import torch
    import paper_2503_05447_amd as pkg
    x = wl.make_inputs(1, 2, 130, 64, 64, kind, dtype="f32", seed=1500 + kind, decay="weak", init_state=True, d_final=True)
    t = to_device(x)
    o, mT, r = run_saved(pkg, t, kind)
    o0, mT0 = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"])
    r0 = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"])
    torch.cuda.synchronize()
    assert torch.equal(o, o0) and torch.equal(mT, mT0)
    for key in ("dq", "dk", "dv", "d_init_state"):
        assert torch.equal(r[key], r0[key]), key
    if kind != wl.KIND_NONE:
        assert torch.equal(r["dg"], r0["dg"])
