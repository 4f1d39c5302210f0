"""Pins of the fp64 oracle against things other than itself (CPU only).

Every pin is something the paper or the mathematics fixes:
  * the unrolled sum M_s = sum_{i<=s} k_i^T v_i and the right-product identity
    (Sec. 2.1.1) -> brute-force quadratic masked form, all four decay kinds;
  * the BLA row of Table 1 -> numpy tril(QK^T)V, a library special case
    (Algorithm 2 with one chunk);
  * the Lightning/RetNet row with constant inputs -> geometric-series closed form;
  * Table 1 caption (scalar is a special vector etc.) -> kind embeddings, bit exact;
  * Algorithm 2 (output = intra + Q * prefix of chunk states, any partition)
    -> carry-over of the state across a split of the sequence;
  * causality of the mask in Algorithm 2; linearity; (b,h) independence;
  * backward: central finite differences of the forward, the closed-form
    gradient of the no-decay case, and the decay-gradient identity.
The paper prints no numeric value for this path, so there is no golden fixture
from the paper itself.
"""
import numpy as np
import pytest

from oracle import (KIND_HEAD, KIND_NONE, KIND_SCALAR, KIND_VECTOR,
                    lsm_oracle_bwd, lsm_oracle_fwd)

KINDS = [KIND_NONE, KIND_HEAD, KIND_SCALAR, KIND_VECTOR]


def rand_case(kind, B=2, H=3, T=23, dk=5, dv=4, seed=0, m0=True, gscale=0.7):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, H, T, dk))
    k = rng.standard_normal((B, H, T, dk))
    v = rng.standard_normal((B, H, T, dv))
    g = {KIND_NONE: None,
         KIND_HEAD: -gscale * rng.random((H,)),
         KIND_SCALAR: -gscale * rng.random((B, H, T)),
         KIND_VECTOR: -gscale * rng.random((B, H, T, dk))}[kind]
    M0 = rng.standard_normal((B, H, dk, dv)) if m0 else None
    return q, k, v, g, M0


def g_full(kind, g, B, H, T, dk):
    """Broadcast any kind's log-decay to [B,H,T,dk] (test-side helper)."""
    if kind == KIND_NONE:
        return np.zeros((B, H, T, dk))
    if kind == KIND_HEAD:
        return np.broadcast_to(g[None, :, None, None], (B, H, T, dk)).copy()
    if kind == KIND_SCALAR:
        return np.broadcast_to(g[..., None], (B, H, T, dk)).copy()
    return g.copy()


def quadratic_form(q, k, v, gf, M0):
    """O = A V + (Q*exp(G)) M0 with A_ts = sum_i q_ti k_si exp(G_ti - G_si), s<=t; brute force."""
    B, H, T, dk = q.shape
    dv = v.shape[-1]
    G = np.cumsum(gf, axis=2)
    o = np.zeros((B, H, T, dv))
    mT = np.zeros((B, H, dk, dv))
    for b in range(B):
        for h in range(H):
            for t in range(T):
                acc = np.zeros(dv)
                for s in range(t + 1):
                    w = np.sum(q[b, h, t] * k[b, h, s] * np.exp(G[b, h, t] - G[b, h, s]))
                    acc += w * v[b, h, s]
                if M0 is not None:
                    acc += (q[b, h, t] * np.exp(G[b, h, t])) @ M0[b, h]
                o[b, h, t] = acc
            m = np.zeros((dk, dv))
            for s in range(T):
                m += np.outer(k[b, h, s] * np.exp(G[b, h, T - 1] - G[b, h, s]), v[b, h, s])
            if M0 is not None:
                m += np.exp(G[b, h, T - 1])[:, None] * M0[b, h]
            mT[b, h] = m
    return o, mT


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("m0", [False, True])
def test_forward_equals_quadratic_masked_form(kind, m0):
    q, k, v, g, M0 = rand_case(kind, m0=m0, seed=11 + kind)
    o, mT = lsm_oracle_fwd(q, k, v, g, kind, M0)
    B, H, T, dk = q.shape
    o2, mT2 = quadratic_form(q, k, v, g_full(kind, g, B, H, T, dk), M0)
    np.testing.assert_allclose(o, o2, rtol=0, atol=1e-11)
    np.testing.assert_allclose(mT, mT2, rtol=0, atol=1e-11)


def test_no_decay_is_tril_matmul():
    q, k, v, _, M0 = rand_case(KIND_NONE, B=1, H=2, T=40, dk=7, dv=6, seed=3)
    o, mT = lsm_oracle_fwd(q, k, v, None, KIND_NONE, M0)
    for h in range(2):
        ref = np.tril(q[0, h] @ k[0, h].T) @ v[0, h] + q[0, h] @ M0[0, h]
        np.testing.assert_allclose(o[0, h], ref, atol=1e-11)
        np.testing.assert_allclose(mT[0, h], M0[0, h] + k[0, h].T @ v[0, h], atol=1e-11)


@pytest.mark.parametrize("kind", [KIND_HEAD, KIND_SCALAR, KIND_VECTOR])
def test_constant_input_closed_form(kind):
    """q=k=1, v=1, constant a:  o_t[j] = dk (1-a^t)/(1-a) + a^t (q M0)[j];  M_T likewise."""
    B, H, T, dk, dv = 1, 2, 37, 6, 3
    a = np.array([0.9, 0.5])
    q = np.ones((B, H, T, dk)); k = np.ones((B, H, T, dk)); v = np.ones((B, H, T, dv))
    gh = np.log(a)
    g = {KIND_HEAD: gh, KIND_SCALAR: np.broadcast_to(gh[None, :, None], (B, H, T)).copy(),
         KIND_VECTOR: np.broadcast_to(gh[None, :, None, None], (B, H, T, dk)).copy()}[kind]
    M0 = np.random.default_rng(5).standard_normal((B, H, dk, dv))
    o, mT = lsm_oracle_fwd(q, k, v, g, kind, M0)
    t = np.arange(1, T + 1)
    for h in range(H):
        geo = (1 - a[h] ** t) / (1 - a[h])
        ref = dk * geo[:, None] + (a[h] ** t)[:, None] * M0[0, h].sum(0)[None, :]
        np.testing.assert_allclose(o[0, h], ref, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(mT[0, h], geo[-1] + a[h] ** T * M0[0, h], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("kind", KINDS)
def test_single_token(kind):
    q, k, v, g, M0 = rand_case(kind, T=1, seed=21)
    o, mT = lsm_oracle_fwd(q, k, v, g, kind, M0)
    B, H, T, dk = q.shape
    a = np.exp(g_full(kind, g, B, H, T, dk))[:, :, 0]                      # [B,H,dk]
    M1 = a[..., None] * M0 + k[:, :, 0, :, None] * v[:, :, 0, None, :]
    np.testing.assert_allclose(mT, M1, atol=1e-13)
    np.testing.assert_allclose(o[:, :, 0], np.einsum("bhi,bhij->bhj", q[:, :, 0], M1), atol=1e-12)


def test_kind_embeddings_are_bit_exact():
    q, k, v, gh, M0 = rand_case(KIND_HEAD, seed=31)
    B, H, T, dk = q.shape
    o_h, m_h = lsm_oracle_fwd(q, k, v, gh, KIND_HEAD, M0)
    gs = np.broadcast_to(gh[None, :, None], (B, H, T)).copy()
    o_s, m_s = lsm_oracle_fwd(q, k, v, gs, KIND_SCALAR, M0)
    gv = np.broadcast_to(gs[..., None], (B, H, T, dk)).copy()
    o_v, m_v = lsm_oracle_fwd(q, k, v, gv, KIND_VECTOR, M0)
    assert np.array_equal(o_h, o_s) and np.array_equal(o_s, o_v)
    assert np.array_equal(m_h, m_s) and np.array_equal(m_s, m_v)
    o_n, m_n = lsm_oracle_fwd(q, k, v, None, KIND_NONE, M0)
    o_z, m_z = lsm_oracle_fwd(q, k, v, np.zeros((B, H, T)), KIND_SCALAR, M0)
    assert np.array_equal(o_n, o_z) and np.array_equal(m_n, m_z)
    # backward embeds the same way (dg sums over the broadcast axes)
    d_o = np.random.default_rng(1).standard_normal(o_h.shape)
    d_m = np.random.default_rng(2).standard_normal(m_h.shape)
    r_h = lsm_oracle_bwd(q, k, v, gh, KIND_HEAD, d_o, M0, d_m)
    r_s = lsm_oracle_bwd(q, k, v, gs, KIND_SCALAR, d_o, M0, d_m)
    r_v = lsm_oracle_bwd(q, k, v, gv, KIND_VECTOR, d_o, M0, d_m)
    for key in ("dq", "dk", "dv", "d_m0"):
        assert np.array_equal(r_h[key], r_s[key]) and np.array_equal(r_s[key], r_v[key])
    np.testing.assert_allclose(r_s["dg"], r_v["dg"].sum(-1), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(r_h["dg"], r_s["dg"].sum((0, 2)), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("split", [1, 9, 22])
def test_state_carry_over_across_a_split(kind, split):
    q, k, v, g, M0 = rand_case(kind, seed=41 + kind)
    o, mT = lsm_oracle_fwd(q, k, v, g, kind, M0)
    sl = lambda x, a, b: None if x is None else (x if kind == KIND_HEAD else x[:, :, a:b])
    T = q.shape[2]
    o1, m1 = lsm_oracle_fwd(q[:, :, :split], k[:, :, :split], v[:, :, :split], sl(g, 0, split), kind, M0)
    o2, m2 = lsm_oracle_fwd(q[:, :, split:], k[:, :, split:], v[:, :, split:], sl(g, split, T), kind, m1)
    assert np.array_equal(np.concatenate([o1, o2], 2), o)       # same operations in the same order
    assert np.array_equal(m2, mT)
    # backward composes through d_mT / d_m0
    rng = np.random.default_rng(7)
    d_o = rng.standard_normal(o.shape); d_m = rng.standard_normal(mT.shape)
    full = lsm_oracle_bwd(q, k, v, g, kind, d_o, M0, d_m)
    second = lsm_oracle_bwd(q[:, :, split:], k[:, :, split:], v[:, :, split:], sl(g, split, T), kind,
                            d_o[:, :, split:], m1, d_m)
    first = lsm_oracle_bwd(q[:, :, :split], k[:, :, :split], v[:, :, :split], sl(g, 0, split), kind,
                           d_o[:, :, :split], M0, second["d_m0"])
    for key in ("dq", "dk", "dv"):
        np.testing.assert_allclose(np.concatenate([first[key], second[key]], 2), full[key], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(first["d_m0"], full["d_m0"], rtol=1e-12, atol=1e-12)
    if kind in (KIND_SCALAR, KIND_VECTOR):
        np.testing.assert_allclose(np.concatenate([first["dg"], second["dg"]], 2), full["dg"], rtol=1e-11, atol=1e-11)
    elif kind == KIND_HEAD:
        np.testing.assert_allclose(first["dg"] + second["dg"], full["dg"], rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("kind", KINDS)
def test_causality_linearity_and_head_independence(kind):
    q, k, v, g, M0 = rand_case(kind, seed=51)
    o, mT = lsm_oracle_fwd(q, k, v, g, kind, M0)
    t = 13
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[:, :, t] += 1.0; v2[:, :, t] -= 2.0; q2[:, :, t] *= 3.0
    o2, _ = lsm_oracle_fwd(q2, k2, v2, g, kind, M0)
    assert np.array_equal(o2[:, :, :t], o[:, :, :t])            # the past does not see token t
    assert not np.array_equal(o2[:, :, t], o[:, :, t])
    # linear in v and in q when M0 = 0
    oa, ma = lsm_oracle_fwd(q, k, v, g, kind, None)
    ob, mb = lsm_oracle_fwd(2.5 * q, k, -0.5 * v, g, kind, None)
    np.testing.assert_allclose(ob, -1.25 * oa, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(mb, -0.5 * ma, rtol=1e-12, atol=1e-12)
    # permuting heads permutes outputs
    perm = [2, 0, 1]
    gp = g if g is None else (g[perm] if kind == KIND_HEAD else g[:, perm])
    op, mp = lsm_oracle_fwd(q[:, perm], k[:, perm], v[:, perm], gp, kind, M0[:, perm])
    assert np.array_equal(op, o[:, perm]) and np.array_equal(mp, mT[:, perm])


def _loss(q, k, v, g, kind, M0, d_o, d_m):
    o, mT = lsm_oracle_fwd(q, k, v, g, kind, M0)
    return float(np.sum(o * d_o) + np.sum(mT * d_m))


@pytest.mark.parametrize("kind", KINDS)
def test_backward_matches_central_differences(kind):
    q, k, v, g, M0 = rand_case(kind, B=1, H=2, T=70, dk=3, dv=4, seed=61 + kind, gscale=0.5)  # 70 > oracle window
    rng = np.random.default_rng(99)
    d_o = rng.standard_normal(v.shape); d_m = rng.standard_normal(M0.shape)
    r = lsm_oracle_bwd(q, k, v, g, kind, d_o, M0, d_m)
    eps = 1e-6
    tensors = dict(q=(q, r["dq"]), k=(k, r["dk"]), v=(v, r["dv"]), M0=(M0, r["d_m0"]))
    if g is not None:
        tensors["g"] = (g, r["dg"])
    probe = np.random.default_rng(5)
    for name, (x, grad) in tensors.items():
        idxs = [tuple(probe.integers(0, s) for s in x.shape) for _ in range(25)]
        # make sure the first and last token are probed too
        if x.ndim >= 3 and name != "M0":
            idxs += [tuple([0, 0, 0] + [0] * (x.ndim - 3)), tuple([0, 1, x.shape[2] - 1] + [0] * (x.ndim - 3))]
        for idx in idxs:
            old = x[idx]
            x[idx] = old + eps; lp = _loss(q, k, v, g, kind, M0, d_o, d_m)
            x[idx] = old - eps; lm = _loss(q, k, v, g, kind, M0, d_o, d_m)
            x[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


def test_backward_no_decay_closed_form():
    q, k, v, _, M0 = rand_case(KIND_NONE, B=1, H=1, T=33, dk=4, dv=5, seed=71)
    rng = np.random.default_rng(8)
    d_o = rng.standard_normal(v.shape); d_m = rng.standard_normal(M0.shape)
    r = lsm_oracle_bwd(q, k, v, None, KIND_NONE, d_o, M0, d_m)
    Q, K, V, dO, m0, dm = q[0, 0], k[0, 0], v[0, 0], d_o[0, 0], M0[0, 0], d_m[0, 0]
    dA = np.tril(dO @ V.T)
    np.testing.assert_allclose(r["dq"][0, 0], dA @ K + dO @ m0.T, atol=1e-11)
    np.testing.assert_allclose(r["dk"][0, 0], dA.T @ Q + V @ dm.T, atol=1e-11)
    np.testing.assert_allclose(r["dv"][0, 0], np.tril(Q @ K.T).T @ dO + K @ dm, atol=1e-11)
    np.testing.assert_allclose(r["d_m0"][0, 0], Q.T @ dO + dm, atol=1e-11)
    assert r["dg"] is None


@pytest.mark.parametrize("kind", [KIND_SCALAR, KIND_VECTOR])
def test_decay_gradient_identity(kind):
    """dg_t = sum_{u>=t} (q_u*dq_u - k_u*dk_u) + rowsum(dM_T * M_T): an independent route to dg."""
    q, k, v, g, M0 = rand_case(kind, B=1, H=2, T=45, dk=4, dv=3, seed=81)
    rng = np.random.default_rng(9)
    d_o = rng.standard_normal(v.shape); d_m = rng.standard_normal(M0.shape)
    r = lsm_oracle_bwd(q, k, v, g, kind, d_o, M0, d_m)
    _, mT = lsm_oracle_fwd(q, k, v, g, kind, M0)
    per = q * r["dq"] - k * r["dk"]                                  # [B,H,T,dk]
    rev = np.flip(np.cumsum(np.flip(per, 2), 2), 2) + np.sum(d_m * mT, -1)[:, :, None, :]
    if kind == KIND_SCALAR:
        rev = rev.sum(-1)
    np.testing.assert_allclose(r["dg"], rev, rtol=1e-10, atol=1e-10)


def test_strong_decay_underflows_harmlessly():
    q, k, v, _, M0 = rand_case(KIND_VECTOR, seed=91)
    B, H, T, dk = q.shape
    g = -800.0 * np.random.default_rng(3).random((B, H, T, dk))      # exp underflows to exact 0
    o, mT = lsm_oracle_fwd(q, k, v, g, KIND_VECTOR, M0)
    assert np.isfinite(o).all() and np.isfinite(mT).all()
    r = lsm_oracle_bwd(q, k, v, g, KIND_VECTOR, np.ones_like(o), M0, None)
    assert all(np.isfinite(x).all() for x in r.values())


def test_argument_validation():
    q, k, v, g, M0 = rand_case(KIND_SCALAR)
    with pytest.raises(ValueError):
        lsm_oracle_fwd(q, k[:, :, :-1], v, g, KIND_SCALAR, M0)
    with pytest.raises(ValueError):
        lsm_oracle_fwd(q, k, v, g[:, :, :-1], KIND_SCALAR, M0)
