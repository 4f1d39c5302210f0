"""Token-major layout and packed variable-length input: both only change where the kernels find their
rows, so the results must be BIT-identical to the head-major / one-call-per-sequence results (which the
other GPU tests compare with the oracle); one packed case is also compared with the oracle directly."""
import numpy as np
import pytest

import lsm_workloads as wl
from lsm_testlib import TOL, host, rel_err, to_device, check

pytestmark = pytest.mark.gpu

KINDS = [wl.KIND_NONE, wl.KIND_HEAD, wl.KIND_SCALAR, wl.KIND_VECTOR]
CASES = [("bf16", 128, 128), ("bf16", 128, 256), ("f32", 64, 64)]   # matrix-core kernels (both), generic kernels


def tm(t, kind=None):
    """[B,H,T,...] -> [B,T,H,...] contiguous (None and per-head decays pass through)."""
    if t is None or t.dim() < 3:
        return t
    return t.transpose(1, 2).contiguous()


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("case", CASES)
def test_token_major_layout_is_bit_identical(kind, case):
    import torch
    import paper_2503_05447_amd as pkg
    dtype, dk, dv = case
    x = wl.make_inputs(2, 3, 150, dk, dv, kind, dtype=dtype, seed=910 + kind, decay="weak", init_state=True, d_final=True)
    t = to_device(x)
    g = t["g"]
    o0, m0 = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], g, kind, 64, t["m0"])
    r0 = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], g, kind, t["d_o"], 64, t["m0"], t["d_mT"])
    g1 = g if kind in (wl.KIND_NONE, wl.KIND_HEAD) else tm(g)
    o1, m1 = pkg.lsm_chunk_fwd(tm(t["q"]), tm(t["k"]), tm(t["v"]), g1, kind, 64, t["m0"], layout=pkg.LAYOUT_BTHD)
    r1 = pkg.lsm_chunk_bwd(tm(t["q"]), tm(t["k"]), tm(t["v"]), g1, kind, tm(t["d_o"]), 64, t["m0"], t["d_mT"],
                           layout=pkg.LAYOUT_BTHD)
    torch.cuda.synchronize()
    assert torch.equal(tm(o1), o0) and torch.equal(m1, m0)
    for key in ("dq", "dk", "dv"):
        assert torch.equal(tm(r1[key]), r0[key]), key
    assert torch.equal(r1["d_init_state"], r0["d_init_state"])
    if kind in (wl.KIND_SCALAR, wl.KIND_VECTOR):
        assert torch.equal(tm(r1["dg"]), r0["dg"])
    elif kind == wl.KIND_HEAD:
        assert torch.equal(r1["dg"], r0["dg"])


LENS = [70, 1, 130, 64, 5]


def packed_case(kind, dtype, dk, dv, H=2, seed=0):
    """One seeded [1,H,T,d] case and its split into sequences of LENS tokens."""
    T = sum(LENS)
    x = wl.make_inputs(1, H, T, dk, dv, kind, dtype=dtype, seed=seed, decay="weak")
    rng = np.random.default_rng(seed + 1)
    n = len(LENS)
    x["m0"] = (rng.standard_normal((n, H, dk, dv)) * 0.1).astype(np.float32)
    x["d_mT"] = (rng.standard_normal((n, H, dk, dv)) * 0.1).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(LENS)]).astype(np.int32)
    return x, cu


def piece(a, lo, hi):
    return None if a is None else a[:, :, lo:hi].contiguous()


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("case", CASES)
def test_packed_sequences_equal_separate_calls(kind, case, layout):
    import torch
    import paper_2503_05447_amd as pkg
    dtype, dk, dv = case
    x, cu = packed_case(kind, dtype, dk, dv, seed=930 + kind)
    t = to_device(x)
    cu_d = torch.from_numpy(cu).to(t["q"].device)
    per_tok = kind in (wl.KIND_SCALAR, wl.KIND_VECTOR)
    L = (lambda a: tm(a)) if layout else (lambda a: a)
    gp = L(t["g"]) if per_tok else t["g"]
    o, mT = pkg.lsm_chunk_fwd(L(t["q"]), L(t["k"]), L(t["v"]), gp, kind, 64, t["m0"], layout=layout, cu_seqlens=cu_d)
    r = pkg.lsm_chunk_bwd(L(t["q"]), L(t["k"]), L(t["v"]), gp, kind, L(t["d_o"]), 64, t["m0"], t["d_mT"], layout=layout,
                          cu_seqlens=cu_d)
    torch.cuda.synchronize()
    if layout:
        o = tm(o)
        r = {k_: (tm(v_) if (v_ is not None and v_.dim() >= 3 and k_ not in ("d_init_state",)) else v_) for k_, v_ in r.items()}
    dg_head = 0
    for s, (lo, hi) in enumerate(zip(cu[:-1], cu[1:])):
        gs = piece(t["g"], lo, hi) if per_tok else t["g"]
        m0s, dms = t["m0"][s:s + 1].contiguous(), t["d_mT"][s:s + 1].contiguous()
        o_s, mT_s = pkg.lsm_chunk_fwd(piece(t["q"], lo, hi), piece(t["k"], lo, hi), piece(t["v"], lo, hi), gs, kind, 64, m0s)
        r_s = pkg.lsm_chunk_bwd(piece(t["q"], lo, hi), piece(t["k"], lo, hi), piece(t["v"], lo, hi), gs, kind,
                                piece(t["d_o"], lo, hi), 64, m0s, dms)
        torch.cuda.synchronize()
        assert torch.equal(o[:, :, lo:hi], o_s), ("o", s)
        assert torch.equal(mT[s:s + 1], mT_s), ("final_state", s)
        for key in ("dq", "dk", "dv"):
            assert torch.equal(r[key][:, :, lo:hi], r_s[key]), (key, s)
        assert torch.equal(r["d_init_state"][s:s + 1], r_s["d_init_state"]), ("d_init_state", s)
        if per_tok:
            assert torch.equal(r["dg"][:, :, lo:hi], r_s["dg"]), ("dg", s)
        elif kind == wl.KIND_HEAD:
            dg_head = dg_head + r_s["dg"]
    if kind == wl.KIND_HEAD:   # one value per head: the packed call sums over all sequences (another summation order)
        assert rel_err(host(r["dg"]), host(dg_head)) <= 1e-4


@pytest.mark.parametrize("kind", [wl.KIND_SCALAR, wl.KIND_VECTOR])
def test_packed_sequences_against_oracle(kind):
    """The oracle of a packed batch is the oracle run on every sequence by itself."""
    import torch
    import paper_2503_05447_amd as pkg
    from oracle import lsm_oracle_bwd, lsm_oracle_fwd
    x, cu = packed_case(kind, "bf16", 128, 128, seed=950 + kind)
    t = to_device(x)
    cu_d = torch.from_numpy(cu).to(t["q"].device)
    o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"], cu_seqlens=cu_d)
    r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"], cu_seqlens=cu_d)
    torch.cuda.synchronize()
    ref = {n: [] for n in ("o", "mT", "dq", "dk", "dv", "dg", "d_m0")}
    for s, (lo, hi) in enumerate(zip(cu[:-1], cu[1:])):
        cut = lambda a: np.ascontiguousarray(a[:, :, lo:hi])
        o_s, mT_s = lsm_oracle_fwd(cut(x["q"]), cut(x["k"]), cut(x["v"]), cut(x["g"]), kind, x["m0"][s:s + 1])
        r_s = lsm_oracle_bwd(cut(x["q"]), cut(x["k"]), cut(x["v"]), cut(x["g"]), kind, cut(x["d_o"]), x["m0"][s:s + 1],
                             x["d_mT"][s:s + 1])
        ref["o"].append(o_s); ref["mT"].append(mT_s)
        for n in ("dq", "dk", "dv", "dg"):
            ref[n].append(r_s[n])
        ref["d_m0"].append(r_s["d_m0"])
    cat_t = lambda n: np.concatenate(ref[n], axis=2)
    check("o", host(o), cat_t("o"), "bf16")
    check("final_state", host(mT), np.concatenate(ref["mT"], axis=0), "bf16")
    for n in ("dq", "dk", "dv"):
        check(n, host(r[n]), cat_t(n), "bf16")
    check("dg", host(r["dg"]), cat_t("dg"), "bf16")
    check("d_init_state", host(r["d_init_state"]), np.concatenate(ref["d_m0"], axis=0), "bf16")


@pytest.mark.parametrize("case", [("bf16", wl.KIND_SCALAR, 128, 128), ("bf16", wl.KIND_SCALAR, 128, 256), ("bf16", wl.KIND_VECTOR, 128, 256),
                                  ("f32", wl.KIND_SCALAR, 64, 64)])
def test_packed_input_with_an_empty_sequence(case):
    """A sequence of length zero passes its initial state (and the gradient of its final state) through."""
    import torch
    import paper_2503_05447_amd as pkg
    dtype, kind, dk, dv = case
    lens = [70, 0, 33]
    T, H, n = sum(lens), 2, len(lens)
    x = wl.make_inputs(1, H, T, dk, dv, kind, dtype=dtype, seed=970, decay="weak")
    rng = np.random.default_rng(971)
    x["m0"] = (rng.standard_normal((n, H, dk, dv)) * 0.1).astype(np.float32)
    x["d_mT"] = (rng.standard_normal((n, H, dk, dv)) * 0.1).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    t = to_device(x)
    cu_d = torch.from_numpy(cu).to(t["q"].device)
    o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"], cu_seqlens=cu_d)
    r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"], cu_seqlens=cu_d)
    torch.cuda.synchronize()
    assert torch.equal(mT[1], t["m0"][1]) and torch.equal(r["d_init_state"][1], t["d_mT"][1])
    for s_, (lo, hi) in enumerate(zip(cu[:-1], cu[1:])):
        if hi == lo:
            continue
        m0s, dms = t["m0"][s_:s_ + 1].contiguous(), t["d_mT"][s_:s_ + 1].contiguous()
        o_s, mT_s = pkg.lsm_chunk_fwd(piece(t["q"], lo, hi), piece(t["k"], lo, hi), piece(t["v"], lo, hi), piece(t["g"], lo, hi),
                                      kind, 64, m0s)
        r_s = pkg.lsm_chunk_bwd(piece(t["q"], lo, hi), piece(t["k"], lo, hi), piece(t["v"], lo, hi), piece(t["g"], lo, hi), kind,
                                piece(t["d_o"], lo, hi), 64, m0s, dms)
        torch.cuda.synchronize()
        assert torch.equal(o[:, :, lo:hi], o_s) and torch.equal(mT[s_:s_ + 1], mT_s)
        for key in ("dq", "dk", "dv", "dg"):
            assert torch.equal(r[key][:, :, lo:hi], r_s[key]), key
        assert torch.equal(r["d_init_state"][s_:s_ + 1], r_s["d_init_state"])
