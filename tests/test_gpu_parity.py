"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element,
on seeded inputs; sizes span several chunks and a ragged tail.  Tolerances: max|x-ref|/RMS(ref)
<= 1e-4 for fp32 inputs, <= 2e-2 for bf16 inputs (fp32 accumulation), per output tensor."""
import numpy as np
import pytest

import lsm_workloads as wl
from lsm_testlib import (check, compare_case, gpu_backward, gpu_forward, host, rel_err, to_device, TOL)

pytestmark = pytest.mark.gpu

KINDS = [wl.KIND_NONE, wl.KIND_HEAD, wl.KIND_SCALAR, wl.KIND_VECTOR]

# (B, H, T, dk, dv, chunk)
SHAPES = [
    (1, 2, 200, 64, 64, 64),      # three chunks and a ragged tail of 8
    (2, 2, 130, 128, 128, 64),    # tail of 2
    (1, 2, 40, 64, 128, 64),      # T < chunk
    (1, 1, 257, 128, 256, 128),   # chunk 128, tail of 1, d_v = 256
    (1, 2, 100, 64, 64, 16),      # chunk 16
    (1, 1, 96, 256, 64, 32),      # chunk 32, d_k = 256, exact multiple
    (1, 2, 150, 128, 256, 64),    # two 128-wide value slices (vector kind: matrix-core path), tail of 22
    (3, 3, 100, 128, 128, 64),    # B*H = 9: not a multiple of the 8 XCDs (tail of the workgroup-id decoding)
]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_parity_weak_decay_with_states(kind, dtype, shape):
    B, H, T, dk, dv, C = shape
    x = wl.make_inputs(B, H, T, dk, dv, kind, dtype=dtype, seed=100 + kind, decay="weak", init_state=True, d_final=True)
    rep = compare_case(x, C)
    print(rep)


@pytest.mark.parametrize("kind", [wl.KIND_HEAD, wl.KIND_SCALAR, wl.KIND_VECTOR])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("decay", ["default", "harsh", "strong4"])
def test_parity_strong_decay_no_states(kind, dtype, decay):
    x = wl.make_inputs(2, 2, 300, 128, 128, kind, dtype=dtype, seed=200 + kind, decay=decay)
    rep = compare_case(x, 64)
    print(rep)


@pytest.mark.parametrize("kind", KINDS)
def test_single_token_and_tiny_sequences(kind):
    for T in (1, 2, 17):
        x = wl.make_inputs(1, 2, T, 64, 64, kind, dtype="f32", seed=300 + T, decay="weak", init_state=True, d_final=True)
        compare_case(x, 16)
        x = wl.make_inputs(1, 2, T, 128, 128, kind, dtype="bf16", seed=300 + T, decay="weak", init_state=True, d_final=True)
        compare_case(x, 64)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chunk_size_independence(kind, dtype):
    import torch
    x = wl.make_inputs(1, 2, 300, 128, 128, kind, dtype=dtype, seed=400 + kind, decay="weak", init_state=True, d_final=True)
    t = to_device(x)
    outs = {}
    for C in (16, 32, 64, 128):
        o, mT = gpu_forward(x, C, t)
        r = gpu_backward(x, C, t)
        torch.cuda.synchronize()
        outs[C] = dict(o=host(o), mT=host(mT), dq=host(r["dq"]), dk=host(r["dk"]), dv=host(r["dv"]),
                       d0=host(r["d_init_state"]), dg=host(r["dg"]))
    for C in (16, 32, 128):
        for key, ref in outs[64].items():
            if ref is None:
                continue
            # two bf16-stored results may differ by one ulp of the container
            ulp = 2.0 ** -7 if (dtype == "bf16" and key in ("o", "dq", "dk", "dv")) else 0.0
            assert rel_err(outs[C][key], ref, ulp) <= 2 * TOL[dtype], (C, key)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_state_carry_over_two_halves_equal_whole(kind, dtype):
    import torch
    import paper_2503_05447_amd as pkg
    x = wl.make_inputs(1, 2, 256, 128, 128, kind, dtype=dtype, seed=500 + kind, decay="weak", init_state=True, d_final=True)
    t = to_device(x)
    o, mT = gpu_forward(x, 64, t)
    full = gpu_backward(x, 64, t)
    s = 128
    gs = lambda a, b: t["g"] if (t["g"] is None or kind == wl.KIND_HEAD) else t["g"][:, :, a:b].contiguous()
    cut = lambda n, a, b: t[n][:, :, a:b].contiguous()
    o1, m1 = pkg.lsm_chunk_fwd(cut("q", 0, s), cut("k", 0, s), cut("v", 0, s), gs(0, s), kind, 64, t["m0"])
    o2, m2 = pkg.lsm_chunk_fwd(cut("q", s, 256), cut("k", s, 256), cut("v", s, 256), gs(s, 256), kind, 64, m1)
    r2 = pkg.lsm_chunk_bwd(cut("q", s, 256), cut("k", s, 256), cut("v", s, 256), gs(s, 256), kind, cut("d_o", s, 256), 64,
                           m1, t["d_mT"])
    r1 = pkg.lsm_chunk_bwd(cut("q", 0, s), cut("k", 0, s), cut("v", 0, s), gs(0, s), kind, cut("d_o", 0, s), 64,
                           t["m0"], r2["d_init_state"])
    torch.cuda.synchronize()
    tol = 2 * TOL[dtype]
    ulp = 2.0 ** -7 if dtype == "bf16" else 0.0   # two bf16-stored results may differ by one ulp
    assert rel_err(host(torch.cat([o1, o2], 2)), host(o), ulp) <= tol
    assert rel_err(host(m2), host(mT)) <= tol
    for key in ("dq", "dk", "dv"):
        assert rel_err(host(torch.cat([r1[key], r2[key]], 2)), host(full[key]), ulp) <= tol, key
    assert rel_err(host(r1["d_init_state"]), host(full["d_init_state"])) <= tol
    if kind in (wl.KIND_SCALAR, wl.KIND_VECTOR):
        assert rel_err(host(torch.cat([r1["dg"], r2["dg"]], 2)), host(full["dg"])) <= tol
    elif kind == wl.KIND_HEAD:
        assert rel_err(host(r1["dg"] + r2["dg"]), host(full["dg"])) <= tol


@pytest.mark.parametrize("kind", KINDS)
def test_run_to_run_bitwise_determinism_and_optional_outputs(kind):
    import torch
    x = wl.make_inputs(2, 2, 200, 128, 128, kind, dtype="bf16", seed=600 + kind, decay="default", init_state=True)
    t = to_device(x)
    a = gpu_forward(x, 64, t)
    b = gpu_forward(x, 64, t)
    ra = gpu_backward(x, 64, t)
    rb = gpu_backward(x, 64, t)
    # optional outputs switched off must not change the others
    c = gpu_forward(x, 64, t, want_final=False)
    rc = gpu_backward(x, 64, t, want_d_log_decay=False, want_d_init_state=False)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[0], c[0]) and c[1] is None
    for key in ("dq", "dk", "dv", "dg", "d_init_state"):
        if ra[key] is not None:
            assert torch.equal(ra[key], rb[key]), key
    for key in ("dq", "dk", "dv"):
        assert torch.equal(ra[key], rc[key]), key
    assert rc["dg"] is None and rc["d_init_state"] is None


def test_kind_embeddings_on_gpu():
    import torch
    x = wl.make_inputs(2, 3, 150, 64, 64, wl.KIND_HEAD, dtype="f32", seed=700, decay="weak", init_state=True, d_final=True)
    t = to_device(x)
    o_h, m_h = gpu_forward(x, 32, t)
    r_h = gpu_backward(x, 32, t)
    xs = dict(x); xs["kind"] = wl.KIND_SCALAR
    xs["g"] = np.ascontiguousarray(np.broadcast_to(x["g"][None, :, None], (2, 3, 150)))
    o_s, m_s = gpu_forward(xs, 32)
    r_s = gpu_backward(xs, 32)
    xv = dict(x); xv["kind"] = wl.KIND_VECTOR
    xv["g"] = np.ascontiguousarray(np.broadcast_to(x["g"][None, :, None, None], (2, 3, 150, 64)))
    o_v, m_v = gpu_forward(xv, 32)
    r_v = gpu_backward(xv, 32)
    torch.cuda.synchronize()
    for a, b in ((o_h, o_s), (o_h, o_v), (m_h, m_s), (m_h, m_v), (r_h["dq"], r_s["dq"]), (r_h["dk"], r_v["dk"]),
                 (r_h["dv"], r_v["dv"])):
        assert rel_err(host(a), host(b)) <= 1e-4
    assert rel_err(host(r_s["dg"]).sum((0, 2)), host(r_h["dg"])) <= 1e-4
    assert rel_err(host(r_v["dg"]).sum(-1), host(r_s["dg"])) <= 1e-4


@pytest.mark.parametrize("case", [("bf16", 128), ("f32", 64)])
def test_largest_batch_times_heads(case):
    """B * H = 65535, the largest the grids allow (the ABI rejects more), short sequences: a sample of
    (b,h) pairs against the oracle, the rest must at least be finite."""
    import torch
    from lsm_testlib import oracle_all, select_heads
    dtype, dd = case
    B, H, T = 255, 257, 3
    x = wl.make_inputs(B, H, T, dd, dd, wl.KIND_SCALAR, dtype=dtype, seed=77, decay="weak", init_state=True, d_final=True)
    t = to_device(x)
    o, mT = gpu_forward(x, 64, t)
    r = gpu_backward(x, 64, t)
    torch.cuda.synchronize()
    for a in (o, mT, r["dq"], r["dk"], r["dv"], r["dg"], r["d_init_state"]):
        assert bool(torch.isfinite(a.float()).all())
    pairs = [(0, 0), (131, 200), (254, 256)]
    y = select_heads(x, pairs)
    o_ref, mT_ref, r_ref = oracle_all(y)
    ib, ih = [p[0] for p in pairs], [p[1] for p in pairs]
    pick = lambda a: host(a[ib, ih][None])
    check("o", pick(o), o_ref, dtype)
    check("final_state", pick(mT), mT_ref, dtype)
    for key in ("dq", "dk", "dv", "dg"):
        check(key, pick(r[key]), r_ref[key], dtype)
    check("d_init_state", pick(r["d_init_state"]), r_ref["d_m0"], dtype)
