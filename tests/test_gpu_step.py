"""GPU parity of the recurrent single-token step (lsm_step) against the fp64 oracle: the oracle is the
token-by-token recurrence itself, called with T = 1 and the running state as its initial state."""
import numpy as np
import pytest

import lsm_workloads as wl
from lsm_testlib import TOL, host, rel_err, BF16_HALF_ULP

pytestmark = pytest.mark.gpu

KINDS = [wl.KIND_NONE, wl.KIND_HEAD, wl.KIND_SCALAR, wl.KIND_VECTOR]


def step_decay(x, t):
    g, kind = x["g"], x["kind"]
    if kind == wl.KIND_NONE:
        return None
    if kind == wl.KIND_HEAD:
        return g
    return np.ascontiguousarray(g[:, :, t])


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 64, 64), (1, 2, 128, 128), (2, 2, 128, 256), (1, 1, 256, 64)])
def test_steps_match_oracle_token_by_token(kind, dtype, shape):
    import torch
    import paper_2503_05447_amd as pkg
    from oracle import lsm_oracle_fwd
    B, H, dk, dv = shape
    T = 5
    x = wl.make_inputs(B, H, T, dk, dv, kind, dtype=dtype, seed=800 + kind, decay="weak", init_state=True)
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    state = torch.from_numpy(x["m0"]).to(dev)
    ref_state = x["m0"].astype(np.float64)
    for t in range(T):
        cut = lambda a: np.ascontiguousarray(a[:, :, t])
        g_t = step_decay(x, t)
        q, k, v = (torch.from_numpy(cut(x[n])).to(dev).to(tdt) for n in ("q", "k", "v"))
        g_dev = None if g_t is None else torch.from_numpy(g_t).to(dev)
        o = pkg.lsm_step(q, k, v, g_dev, kind, state)
        torch.cuda.synchronize()
        # oracle: one token from the oracle's own running state
        g_o = None if g_t is None else (g_t if kind == wl.KIND_HEAD else g_t[:, :, None])
        o_ref, ref_state = lsm_oracle_fwd(x["q"][:, :, t:t + 1], x["k"][:, :, t:t + 1], x["v"][:, :, t:t + 1], g_o, kind,
                                          ref_state.astype(np.float32))
        ulp = BF16_HALF_ULP if dtype == "bf16" else 0.0
        assert rel_err(host(o), o_ref[:, :, 0], ulp) <= TOL[dtype], ("o", t)
        # the oracle restarts from the fp32 copy of its state each token: compare at fp32 granularity
        assert rel_err(host(state), ref_state) <= (1e-5 if dtype == "f32" else TOL[dtype]), ("state", t)
        ref_state = host(state)   # keep both on the same trajectory; each step is checked on its own


@pytest.mark.parametrize("kind", KINDS)
def test_steps_equal_chunked_forward(kind):
    """T recurrent steps from init_state = the chunkwise forward over the same T tokens (Algorithm 2 vs Eq. 5)."""
    import torch
    import paper_2503_05447_amd as pkg
    from lsm_testlib import to_device
    B, H, T, dk, dv = 2, 2, 70, 128, 128
    x = wl.make_inputs(B, H, T, dk, dv, kind, dtype="bf16", seed=850 + kind, decay="weak", init_state=True)
    t = to_device(x)
    o_chunk, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"])
    state = t["m0"].clone()
    outs = []
    for s in range(T):
        g = None if t["g"] is None else (t["g"] if kind == wl.KIND_HEAD else t["g"][:, :, s].contiguous())
        outs.append(pkg.lsm_step(t["q"][:, :, s].contiguous(), t["k"][:, :, s].contiguous(), t["v"][:, :, s].contiguous(),
                                 g, kind, state))
    torch.cuda.synchronize()
    o_step = torch.stack(outs, 2)
    assert rel_err(host(o_chunk), host(o_step), 2.0 ** -7) <= TOL["bf16"]
    assert rel_err(host(mT), host(state)) <= TOL["bf16"]


@pytest.mark.parametrize("gated", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 64, 64), (1, 2, 128, 128), (2, 2, 128, 256), (1, 1, 256, 64)])
def test_delta_rule_steps_match_oracle_token_by_token(shape, dtype, gated):
    """lsm_delta_step against the delta-rule oracle called with T = 1 from its own running state; all three per-token
    parameters present in the gated case."""
    import torch
    import paper_2503_05447_amd as pkg
    from oracle import delta_oracle_fwd
    B, H, dk, dv = shape
    T = 6
    x = wl.make_delta_inputs(B, H, T, dk, dv, gated, dtype=dtype, seed=860 + int(gated), init_state=True, tie_b=False)
    if gated:
        x["beta"] = (0.2 + 0.7 * np.random.default_rng(3).random((B, H, T))).astype(np.float32)
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    state = torch.from_numpy(x["m0"]).to(dev)
    ref_state = x["m0"].astype(np.float64)
    for t in range(T):
        cut = lambda a: None if a is None else np.ascontiguousarray(a[:, :, t])
        q, k, v = (torch.from_numpy(cut(x[n])).to(dev).to(tdt) for n in ("q", "k", "v"))
        par = lambda n: None if x[n] is None else torch.from_numpy(cut(x[n])).to(dev)
        o = pkg.lsm_delta_step(q, k, v, state, par("log_alpha"), par("beta"), par("b"))
        torch.cuda.synchronize()
        sl = lambda a: None if a is None else a[:, :, t:t + 1]
        o_ref, ref_state = delta_oracle_fwd(sl(x["q"]), sl(x["k"]), sl(x["v"]), sl(x["log_alpha"]), sl(x["beta"]), sl(x["b"]),
                                            ref_state.astype(np.float32))
        ulp = BF16_HALF_ULP if dtype == "bf16" else 0.0
        assert rel_err(host(o), o_ref[:, :, 0], ulp) <= TOL[dtype], ("o", t)
        assert rel_err(host(state), ref_state) <= 1e-5, ("state", t)
        ref_state = host(state)   # both sides go on from the same fp32 state


def test_delta_rule_steps_equal_the_chunkwise_forward():
    import torch
    import paper_2503_05447_amd as pkg
    x = wl.make_delta_inputs(1, 2, 70, 128, 128, True, seed=870, init_state=True)
    dev = torch.device("cuda:0")
    mv = lambda a, dt: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt).contiguous()
    q, k, v = (mv(x[n], torch.bfloat16) for n in ("q", "k", "v"))
    la, bw, m0 = (mv(x[n], torch.float32) for n in ("log_alpha", "b", "m0"))
    o_c, m_c = pkg.lsm_delta_fwd(q, k, v, la, None, bw, m0)
    state = m0.clone()
    outs = [pkg.lsm_delta_step(q[:, :, t].contiguous(), k[:, :, t].contiguous(), v[:, :, t].contiguous(), state,
                               la[:, :, t].contiguous(), None, bw[:, :, t].contiguous()) for t in range(70)]
    torch.cuda.synchronize()
    o_s = torch.stack(outs, dim=2)
    assert rel_err(host(o_s), host(o_c)) <= 2e-2
    assert rel_err(host(state), host(m_c)) <= 2e-3
