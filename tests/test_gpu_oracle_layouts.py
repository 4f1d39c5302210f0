"""GPU parity against the fp64 oracle for what earlier tests only compared HIP against HIP, and for the
corners of the segmented chunk walkers:
  * the token-major [B,T,H,d] layout, directly against the oracle (matrix-core scalar and vector kernels,
    generic fp32 kernels), also packed and with the forward call's states kept;
  * strong decays together with a carried-in state and a gradient of the final state;
  * the segment plan of the chunk walkers: many sequences (one segment each), few sequences (many short
    segments, ragged last segment), chunk counts that the segment length does not divide."""
import numpy as np
import pytest

import lsm_workloads as wl
from lsm_testlib import check, host, oracle_all, to_device

pytestmark = pytest.mark.gpu


def tm(t):
    """[B,H,T,...] -> [B,T,H,...] contiguous (None and per-head decays pass through)."""
    if t is None or t.dim() < 3:
        return t
    return t.transpose(1, 2).contiguous()


def compare_token_major(x, chunk=64, saved=False, cu=None):
    """Run the library on the token-major copy of a seeded case; compare every tensor with the oracle."""
    import torch
    import paper_2503_05447_amd as pkg
    t = to_device(x)
    kind = x["kind"]
    per_tok = kind in (wl.KIND_SCALAR, wl.KIND_VECTOR)
    q, k, v, d_o = tm(t["q"]), tm(t["k"]), tm(t["v"]), tm(t["d_o"])
    g = tm(t["g"]) if per_tok else t["g"]
    kw = dict(layout=pkg.LAYOUT_BTHD, cu_seqlens=cu)
    if saved:
        ws = pkg.lsm_chunk_workspace(q, k, v, g, kind, chunk, pkg.LAYOUT_BTHD, cu, save_states=True)
        o, mT = pkg.lsm_chunk_fwd(q, k, v, g, kind, chunk, t["m0"], workspace=ws, save_states=True, **kw)
        r = pkg.lsm_chunk_bwd(q, k, v, g, kind, d_o, chunk, t["m0"], t["d_mT"], workspace=ws, states_saved=True, **kw)
    else:
        o, mT = pkg.lsm_chunk_fwd(q, k, v, g, kind, chunk, t["m0"], **kw)
        r = pkg.lsm_chunk_bwd(q, k, v, g, kind, d_o, chunk, t["m0"], t["d_mT"], **kw)
    torch.cuda.synchronize()
    return tm(o), mT, {n: (tm(a) if n in ("dq", "dk", "dv") or (n == "dg" and per_tok) else a) for n, a in r.items()}


def check_head_dg(x, got, ref):
    """Per-head decay gradient: dg[h] is the sum over all B*T tokens of the per-token gradients a per-token decay
    with the same values would get.  Under a weak decay those are large and cancel (each is of the size of
    <M_t, dM_t>, their sum of the size of a few of them), so the error of the sum is set against what per-token
    errors at the tolerance add up to: tol * max(|ref[h]|, RMS over tokens * sqrt(B*T))."""
    from oracle import lsm_oracle_bwd
    B, H, T = x["B"], x["H"], x["T"]
    g_tok = np.ascontiguousarray(np.broadcast_to(x["g"][None, :, None], (B, H, T))).astype(np.float32)
    per_tok = lsm_oracle_bwd(x["q"], x["k"], x["v"], g_tok, wl.KIND_SCALAR, x["d_o"], x["m0"], x["d_mT"])["dg"]
    assert np.allclose(per_tok.sum(axis=(0, 2)), ref, rtol=1e-9, atol=1e-9 * np.abs(ref).max())   # the same quantity
    scale = np.sqrt(np.mean(per_tok ** 2, axis=(0, 2))) * np.sqrt(B * T)
    tol = {"f32": 1e-4, "bf16": 2e-2}[x["dtype"]]
    assert np.isfinite(got).all()
    bad = np.abs(got - ref) > tol * np.maximum(np.abs(ref), scale)
    assert not bad.any(), (got, ref, scale)


def check_all(x, o, mT, r, ref):
    o_ref, mT_ref, r_ref = ref
    dt = x["dtype"]
    check("o", host(o), o_ref, dt)
    check("final_state", host(mT), mT_ref, dt)
    for n in ("dq", "dk", "dv"):
        check(n, host(r[n]), r_ref[n], dt)
    check("d_init_state", host(r["d_init_state"]), r_ref["d_m0"], dt)
    if x["kind"] == wl.KIND_HEAD:
        check_head_dg(x, host(r["dg"]), r_ref["dg"])
    elif x["kind"] != wl.KIND_NONE:
        check("dg", host(r["dg"]), r_ref["dg"], dt)


CASES = [("bf16", wl.KIND_SCALAR, 128, 128), ("bf16", wl.KIND_HEAD, 128, 128), ("bf16", wl.KIND_NONE, 128, 128),
         ("bf16", wl.KIND_VECTOR, 128, 256), ("f32", wl.KIND_SCALAR, 64, 64), ("f32", wl.KIND_VECTOR, 64, 128)]


@pytest.mark.parametrize("saved", [False, True])
@pytest.mark.parametrize("case", CASES)
def test_token_major_layout_against_oracle(case, saved):
    dtype, kind, dk, dv = case
    x = wl.make_inputs(2, 3, 333, dk, dv, kind, dtype=dtype, seed=2100 + kind, decay="weak", init_state=True, d_final=True)
    o, mT, r = compare_token_major(x, saved=saved)
    check_all(x, o, mT, r, oracle_all(x))


@pytest.mark.parametrize("case", [("bf16", wl.KIND_SCALAR, 128, 128), ("bf16", wl.KIND_VECTOR, 128, 128), ("f32", wl.KIND_HEAD, 64, 64)])
def test_packed_token_major_with_kept_states_against_oracle(case):
    """Packed sequences, token-major, the forward call's states kept: the oracle runs on every sequence by itself."""
    import torch
    from oracle import lsm_oracle_bwd, lsm_oracle_fwd
    dtype, kind, dk, dv = case
    lens = [70, 1, 700, 64, 5]
    T, H, n = sum(lens), 2, len(lens)
    x = wl.make_inputs(1, H, T, dk, dv, kind, dtype=dtype, seed=2200 + kind, decay="weak")
    rng = np.random.default_rng(2201)
    x["m0"] = (rng.standard_normal((n, H, dk, dv)) * 0.1).astype(np.float32)
    x["d_mT"] = (rng.standard_normal((n, H, dk, dv)) * 0.1).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_d = torch.from_numpy(cu).to("cuda:0")
    o, mT, r = compare_token_major(x, saved=True, cu=cu_d)
    per_tok = kind in (wl.KIND_SCALAR, wl.KIND_VECTOR)
    ref = {m: [] for m in ("o", "mT", "dq", "dk", "dv", "dg", "d_m0")}
    for s, (lo, hi) in enumerate(zip(cu[:-1], cu[1:])):
        cut = lambda a: np.ascontiguousarray(a[:, :, lo:hi])
        gs = cut(x["g"]) if per_tok else x["g"]
        o_s, mT_s = lsm_oracle_fwd(cut(x["q"]), cut(x["k"]), cut(x["v"]), gs, kind, x["m0"][s:s + 1])
        r_s = lsm_oracle_bwd(cut(x["q"]), cut(x["k"]), cut(x["v"]), gs, kind, cut(x["d_o"]), x["m0"][s:s + 1], x["d_mT"][s:s + 1])
        ref["o"].append(o_s); ref["mT"].append(mT_s); ref["d_m0"].append(r_s["d_m0"])
        for m in ("dq", "dk", "dv", "dg"):
            ref[m].append(r_s[m])
    cat_t = lambda m: np.concatenate(ref[m], axis=2)
    check("o", host(o), cat_t("o"), dtype)
    check("final_state", host(mT), np.concatenate(ref["mT"], axis=0), dtype)
    for m in ("dq", "dk", "dv"):
        check(m, host(r[m]), cat_t(m), dtype)
    check("d_init_state", host(r["d_init_state"]), np.concatenate(ref["d_m0"], axis=0), dtype)
    dg_ref = cat_t("dg") if per_tok else np.sum(ref["dg"], axis=0)
    check("dg", host(r["dg"]), dg_ref, dtype)


@pytest.mark.parametrize("saved", [False, True])
@pytest.mark.parametrize("decay", ["default", "strong4", "harsh"])
@pytest.mark.parametrize("kind", [wl.KIND_HEAD, wl.KIND_SCALAR, wl.KIND_VECTOR])
def test_strong_decay_with_carried_states(kind, decay, saved):
    """Strong decays with an initial state and a gradient of the final state, on the recomputing and on the
    state-keeping matrix-core path.  The states are drawn at the scale of one token's own k^T v (1 / sqrt(d_k) per
    element of k and v), so that the tokens they reach do not dwarf the RMS of the rest."""
    import torch
    import paper_2503_05447_amd as pkg
    x = wl.make_inputs(2, 2, 300, 128, 128, kind, dtype="bf16", seed=2300 + kind, decay=decay, init_state=True, d_final=True,
                       init_std=1.0 / 128)
    t = to_device(x)
    if saved:
        ws = pkg.lsm_chunk_workspace(t["q"], t["k"], t["v"], t["g"], kind, 64, save_states=True)
        o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"], workspace=ws, save_states=True)
        r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"], workspace=ws,
                              states_saved=True)
    else:
        o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"])
        r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"])
    torch.cuda.synchronize()
    check_all(x, o, mT, r, oracle_all(x))


# (B, H, T): 512 sequences -> one segment each; 6 sequences -> many segments; T chosen so that the last segment and
# the last chunk are both ragged; one chunk only; two sequences with 21 chunks; 40 sequences of 24 chunks -> walker
# segments of two chunks, and a reverse scan in four segments of three walker segments each
SEGMENT_SHAPES = [(32, 16, 130), (2, 3, 1500), (1, 5, 1111), (1, 1, 64), (1, 2, 1300), (5, 8, 1500)]


@pytest.mark.parametrize("saved", [False, True])
@pytest.mark.parametrize("kind", [wl.KIND_NONE, wl.KIND_HEAD, wl.KIND_SCALAR])
@pytest.mark.parametrize("shape", SEGMENT_SHAPES)
def test_segment_plans_of_the_chunk_walkers(kind, shape, saved):
    import torch
    import paper_2503_05447_amd as pkg
    B, H, T = shape
    x = wl.make_inputs(B, H, T, 128, 128, kind, dtype="bf16", seed=2400 + T + kind, decay="weak", init_state=True, d_final=True)
    t = to_device(x)
    if saved:
        ws = pkg.lsm_chunk_workspace(t["q"], t["k"], t["v"], t["g"], kind, 64, save_states=True)
        o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"], workspace=ws, save_states=True)
        r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"], workspace=ws,
                              states_saved=True)
    else:
        o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"])
        r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"])
    torch.cuda.synchronize()
    check_all(x, o, mT, r, oracle_all(x))


# ---- scalar decay kinds with d_v = 256: the matrix-core walkers take one 128-wide value slice per pass; the query,
# key and decay gradients sum over the slices

WIDE_SHAPES = [(2, 3, 333), (1, 2, 1300), (8, 8, 200)]   # a few segments; many chunks; one segment per sequence


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("kind", [wl.KIND_NONE, wl.KIND_HEAD, wl.KIND_SCALAR])
@pytest.mark.parametrize("shape", WIDE_SHAPES)
def test_scalar_kinds_with_wide_values_run_on_the_matrix_cores(shape, kind, layout):
    import torch
    import paper_2503_05447_amd as pkg
    B, H, T = shape
    x = wl.make_inputs(B, H, T, 128, 256, kind, dtype="bf16", seed=2500 + T + kind, decay="weak", init_state=True, d_final=True)
    p = pkg.make_params(B, H, T, 128, 256, 64, kind, 1, layout=layout)
    assert pkg.kernel_path(p) == 1, "bf16, chunk 64, d_k = 128, d_v = 256 must run on the MFMA kernels"
    assert pkg.keeps_states(pkg.make_params(B, H, T, 128, 256, 64, kind, 1, layout=layout, flags=pkg.FLAG_SAVE_STATES)) == 0
    if layout == 1:
        o, mT, r = compare_token_major(x)
    else:
        t = to_device(x)
        # the flag is accepted and changes nothing here: the backward call recomputes
        ws = pkg.lsm_chunk_workspace(t["q"], t["k"], t["v"], t["g"], kind, 64, save_states=True)
        o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], kind, 64, t["m0"], workspace=ws, save_states=True)
        r = pkg.lsm_chunk_bwd(t["q"], t["k"], t["v"], t["g"], kind, t["d_o"], 64, t["m0"], t["d_mT"], workspace=ws,
                              states_saved=True)
        torch.cuda.synchronize()
    check_all(x, o, mT, r, oracle_all(x))


def test_wide_values_equal_two_narrow_calls_in_the_forward():
    """Each 128-wide slice of the values is a recurrence of its own: o and the final state of a d_v = 256 call equal,
    bit for bit, those of two d_v = 128 calls on the halves of v."""
    import torch
    import paper_2503_05447_amd as pkg
    x = wl.make_inputs(2, 2, 700, 128, 256, wl.KIND_SCALAR, dtype="bf16", seed=2601, decay="default", init_state=True)
    t = to_device(x)
    o, mT = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"], t["g"], wl.KIND_SCALAR, 64, t["m0"])
    for s in range(2):
        sl = slice(128 * s, 128 * s + 128)
        o_s, mT_s = pkg.lsm_chunk_fwd(t["q"], t["k"], t["v"][..., sl].contiguous(), t["g"], wl.KIND_SCALAR, 64,
                                      t["m0"][..., sl].contiguous())
        torch.cuda.synchronize()
        assert torch.equal(o[..., sl], o_s) and torch.equal(mT[..., sl], mT_s), s


def test_packed_wide_values_against_oracle():
    import torch
    from oracle import lsm_oracle_bwd, lsm_oracle_fwd
    kind, dk, dv, dtype = wl.KIND_SCALAR, 128, 256, "bf16"
    lens = [70, 1, 700, 64, 5]
    T, H, n = sum(lens), 2, len(lens)
    x = wl.make_inputs(1, H, T, dk, dv, kind, dtype=dtype, seed=2700, decay="weak")
    rng = np.random.default_rng(2701)
    x["m0"] = (rng.standard_normal((n, H, dk, dv)) * 0.1).astype(np.float32)
    x["d_mT"] = (rng.standard_normal((n, H, dk, dv)) * 0.1).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    o, mT, r = compare_token_major(x, cu=torch.from_numpy(cu).to("cuda:0"))
    ref = {m: [] for m in ("o", "mT", "dq", "dk", "dv", "dg", "d_m0")}
    for s, (lo, hi) in enumerate(zip(cu[:-1], cu[1:])):
        cut = lambda a: np.ascontiguousarray(a[:, :, lo:hi])
        o_s, mT_s = lsm_oracle_fwd(cut(x["q"]), cut(x["k"]), cut(x["v"]), cut(x["g"]), kind, x["m0"][s:s + 1])
        r_s = lsm_oracle_bwd(cut(x["q"]), cut(x["k"]), cut(x["v"]), cut(x["g"]), kind, cut(x["d_o"]), x["m0"][s:s + 1], x["d_mT"][s:s + 1])
        ref["o"].append(o_s); ref["mT"].append(mT_s); ref["d_m0"].append(r_s["d_m0"])
        for m in ("dq", "dk", "dv", "dg"):
            ref[m].append(r_s[m])
    cat_t = lambda m: np.concatenate(ref[m], axis=2)
    check("o", host(o), cat_t("o"), dtype)
    check("final_state", host(mT), np.concatenate(ref["mT"], axis=0), dtype)
    for m in ("dq", "dk", "dv", "dg"):
        check(m, host(r[m]), cat_t(m), dtype)
    check("d_init_state", host(r["d_init_state"]), np.concatenate(ref["d_m0"], axis=0), dtype)
