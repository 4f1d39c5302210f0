"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no synchronisation),
so its calls can be recorded into a HIP graph.  Every replay must reproduce the eager results bit for bit,
also with unrelated eager work and synchronisations between the replays."""
import pytest

import lsm_workloads as wl
from lsm_testlib import to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("keep", [False, "always"])
@pytest.mark.parametrize("kind", [wl.KIND_SCALAR, wl.KIND_VECTOR])
def test_forward_backward_replayed_from_a_graph(kind, keep):
    """keep: the forward call leaves its chunk states in the workspace for the backward call."""
    import torch
    import paper_2503_05447_amd as pkg
    x = wl.make_inputs(2, 2, 200, 128, 128, kind, dtype="bf16", seed=990 + kind, decay="weak", init_state=True, d_final=True)
    t = to_device(x)
    ws = pkg.lsm_chunk_workspace(t["q"], t["k"], t["v"], t["g"], kind, save_states=keep)
    run = lambda: (pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"], workspace=ws, save_states=keep),
                   pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"], workspace=ws,
                                     states_saved=keep))
    (o_e, m_e), r_e = run()
    torch.cuda.synchronize()
    eager = [o_e.clone(), m_e.clone()] + [r_e[n].clone() for n in ("dq", "dk", "dv", "dg", "d_init_state")]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()   # warm-up on the capture stream (function attributes are set outside the capture)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        (o_g, m_g), r_g = run()
    outs = [o_g, m_g] + [r_g[n] for n in ("dq", "dk", "dv", "dg", "d_init_state")]
    for rep in range(3):
        for buf in outs:
            buf.fill_(0)   # a fill kernel, eager
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, eager):
            assert torch.equal(got, ref), rep
        (t["q"].float() @ t["k"].float().transpose(-1, -2)).sum().item()   # unrelated eager work in between


def test_decode_steps_replayed_from_a_graph():
    import torch
    import paper_2503_05447_amd as pkg
    B, H, dk, dv, steps = 4, 4, 128, 128, 8
    dev = torch.device("cuda:0")
    g0 = torch.Generator(device=dev).manual_seed(5)
    q = torch.randn(steps, B, H, dk, device=dev, generator=g0).to(torch.bfloat16)
    k = (torch.randn(steps, B, H, dk, device=dev, generator=g0) / dk ** 0.5).to(torch.bfloat16)
    v = torch.randn(steps, B, H, dv, device=dev, generator=g0).to(torch.bfloat16)
    g = -torch.rand(steps, B, H, device=dev, generator=g0)
    state0 = torch.randn(B, H, dk, dv, device=dev, generator=g0)
    def run(state, o):
        for s in range(steps):
            pkg.lsm_step(q[s], k[s], v[s], g[s], wl.KIND_SCALAR, state, o[s])
    st_e, o_e = state0.clone(), torch.empty(steps, B, H, dv, device=dev, dtype=torch.bfloat16)
    run(st_e, o_e)
    torch.cuda.synchronize()
    st_g, o_g = state0.clone(), torch.empty_like(o_e)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(st_g, o_g)
    for rep in range(3):
        st_g.copy_(state0)
        o_g.fill_(0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_g, o_e) and torch.equal(st_g, st_e), rep


@pytest.mark.parametrize("keep", [False, True])
@pytest.mark.parametrize("gated", [False, True])
def test_delta_rule_forward_backward_replayed_from_a_graph(gated, keep):
    import numpy as np
    import torch
    import paper_2503_05447_amd as pkg
    x = wl.make_delta_inputs(2, 2, 200, 128, 128, gated, seed=995 + int(gated), init_state=True, d_final=True)
    dev = torch.device("cuda:0")
    mv = lambda a, dt: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt).contiguous()
    q, k, v, d_o = (mv(x[n], torch.bfloat16) for n in ("q", "k", "v", "d_o"))
    la, be, bw, m0, d_mT = (mv(x[n], torch.float32) for n in ("log_alpha", "beta", "b", "m0", "d_mT"))
    ws = pkg.lsm_delta_workspace(q, k, v, la)
    run = lambda: (pkg.lsm_delta_fwd(q, k, v, la, be, bw, m0, workspace=ws, save_states=keep),
                   pkg.lsm_delta_bwd(q, k, v, d_o, la, be, bw, m0, d_mT, workspace=ws, states_saved=keep))
    names = [n for n in ("dq", "dk", "dv", "d_log_alpha", "d_beta", "d_b", "d_init_state")]
    (o_e, m_e), r_e = run()
    torch.cuda.synchronize()
    eager = [o_e.clone(), m_e.clone()] + [r_e[n].clone() for n in names if r_e[n] is not None]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()   # warm-up on the capture stream (function attributes are set outside the capture)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        (o_g, m_g), r_g = run()
    outs = [o_g, m_g] + [r_g[n] for n in names if r_g[n] is not None]
    for rep in range(3):
        for buf in outs:
            buf.fill_(0)
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, eager):
            assert torch.equal(got, ref), rep
        (q.float() @ k.float().transpose(-1, -2)).sum().item()   # unrelated eager work in between
