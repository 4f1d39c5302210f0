"""Pins of the fp64 delta-rule oracle against things other than itself (CPU only).

What the paper and the mathematics fix for the DeltaNet / Gated DeltaNet rows of Table 1:
  * with a_s = 0 (DeltaNet) the row IS the BLA / Mamba2-style row with values b_s v_s: the independent
    diagonal-decay oracle must agree, forward and backward (Table 1: all rows share Eq. 5);
  * the stored-value property that gives the rule its name: with a unit key and a_s = b_s = 1 the state
    returns exactly v_s when queried with k_s, whatever it held before; orthonormal keys do not disturb each other
    and rewriting a key replaces its value;
  * a block of tokens solved at once: the pseudo-values u_t = b_t v_t - beta_t Gamma_t k_t S - ... of the block
    solve a unit lower-triangular system, handed to scipy's triangular solver (the published chunkwise form of
    the delta rule) -- a different algorithm for the same numbers;
  * the update as one gradient step on l(M) = |k M - v|^2 / 2 (the reading under which Table 1 lists TTT and
    Titans next to it), with the gradient of l taken by finite differences;
  * the Gated DeltaNet row as the product form M_s = a_s P_s M_{s-1} + ..., P_s a projector for a unit key:
    directions along k_s are erased (k_s M_s = b_s v_s), directions orthogonal to it only decay;
  * backward: central finite differences of the forward for every input, linearity in d_o, (b,h) independence.
The paper prints no numeric value for these rows, so there is no golden fixture from the paper itself.
"""
import numpy as np
import pytest
import scipy.linalg

from oracle import KIND_NONE, KIND_SCALAR, delta_oracle_bwd, delta_oracle_fwd, lsm_oracle_bwd, lsm_oracle_fwd


def rand_case(B=2, H=2, T=19, dk=5, dv=4, seed=0, gated=True, unit_keys=True, m0=True):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, H, T, dk))
    k = rng.standard_normal((B, H, T, dk))
    if unit_keys:
        k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((B, H, T, dv))
    la = -0.5 * rng.random((B, H, T)) if gated else None
    beta = 0.1 + 0.8 * rng.random((B, H, T))
    b = 0.2 + rng.random((B, H, T))
    M0 = rng.standard_normal((B, H, dk, dv)) if m0 else None
    return q, k, v, la, beta, b, M0


@pytest.mark.parametrize("gated", [False, True])
def test_zero_a_reduces_to_the_diagonal_decay_rows(gated):
    q, k, v, la, beta, b, M0 = rand_case(seed=3, gated=gated, unit_keys=False)
    rng = np.random.default_rng(4)
    d_o, d_mT = rng.standard_normal(v.shape), rng.standard_normal(M0.shape)
    zero = np.zeros_like(beta)
    o, mT = delta_oracle_fwd(q, k, v, la, zero, b, M0)
    kind = KIND_SCALAR if gated else KIND_NONE
    o_ref, mT_ref = lsm_oracle_fwd(q, k, b[..., None] * v, la, kind, M0)
    np.testing.assert_allclose(o, o_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(mT, mT_ref, rtol=1e-12, atol=1e-12)
    r = delta_oracle_bwd(q, k, v, d_o, la, zero, b, M0, d_mT)
    ref = lsm_oracle_bwd(q, k, b[..., None] * v, la, kind, d_o, M0, d_mT)
    np.testing.assert_allclose(r["dq"], ref["dq"], rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(r["dk"], ref["dk"], rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(r["dv"], b[..., None] * ref["dv"], rtol=1e-11, atol=1e-11)       # chain rule through b v
    np.testing.assert_allclose(r["d_b"], (ref["dv"] * v).sum(-1), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(r["d_m0"], ref["d_m0"], rtol=1e-11, atol=1e-11)
    if gated:
        np.testing.assert_allclose(r["d_log_alpha"], ref["dg"], rtol=1e-11, atol=1e-11)


def test_unit_key_stores_its_value_exactly():
    # DeltaNet row with a_s = b_s = 1: k_s M_s = v_s for every s, whatever M_{s-1} was
    q, k, v, _, _, _, M0 = rand_case(seed=5, gated=False)
    B, H, T, dk = k.shape
    one = np.ones((B, H, T))
    for t in range(1, T + 1):
        # query with the last key of the prefix
        qq = q[:, :, :t].copy()
        qq[:, :, t - 1] = k[:, :, t - 1]
        o, _ = delta_oracle_fwd(qq, k[:, :, :t], v[:, :, :t], None, one[:, :, :t], one[:, :, :t], M0)
        np.testing.assert_allclose(o[:, :, t - 1], v[:, :, t - 1], rtol=1e-12, atol=1e-12)


def test_orthonormal_keys_do_not_interfere_and_rewrites_replace():
    rng = np.random.default_rng(6)
    dk, dv = 6, 3
    Qm, _ = np.linalg.qr(rng.standard_normal((dk, dk)))
    keys = Qm[:4]                                                  # four orthonormal keys
    vals = rng.standard_normal((5, dv))
    k = np.concatenate([keys, keys[1:2]])[None, None]              # the fifth token rewrites key 1
    v = vals[None, None]
    one = np.ones((1, 1, 5))
    _, mT = delta_oracle_fwd(k, k, v, None, one, one, None)
    want = keys[0][:, None] * vals[0] + keys[1][:, None] * vals[4] + keys[2][:, None] * vals[2] + keys[3][:, None] * vals[3]
    np.testing.assert_allclose(mT[0, 0], want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("gated", [False, True])
def test_block_of_tokens_by_triangular_solve(gated):
    # With Gamma_t = prod_{s<=t} alpha_s inside the block and S the state before it:
    #   M_t = alpha_t M_{t-1} + k_t^T u_t ,  u_t = b_t v_t - beta_t Gamma_t k_t S - beta_t sum_{r<t} (Gamma_t/Gamma_r)(k_t.k_r) u_r
    # i.e. (I + L) U = diag(b) V - diag(beta Gamma) K S with L strictly lower triangular, and then
    #   o_t = Gamma_t q_t S + sum_{r<=t} (Gamma_t/Gamma_r)(q_t.k_r) u_r ,  M_end = Gamma_C S + sum_r (Gamma_C/Gamma_r) k_r^T u_r .
    q, k, v, la, beta, b, M0 = rand_case(B=1, H=2, T=37, dk=6, dv=5, seed=7, gated=gated, unit_keys=False)
    k *= 0.6
    o, mT = delta_oracle_fwd(q, k, v, la, beta, b, M0)
    for h in range(2):
        S = M0[0, h].copy()
        for t0 in range(0, 37, 16):                              # blocks of 16, the last one ragged
            sl = slice(t0, min(t0 + 16, 37))
            Q, K, V, be, bb = q[0, h, sl], k[0, h, sl], v[0, h, sl], beta[0, h, sl], b[0, h, sl]
            lg = np.cumsum(la[0, h, sl]) if gated else np.zeros(len(be))
            D = np.exp(lg[:, None] - lg[None, :])                 # Gamma_t / Gamma_r
            L = np.tril(be[:, None] * D * (K @ K.T), -1)
            rhs = bb[:, None] * V - (be * np.exp(lg))[:, None] * (K @ S)
            U = scipy.linalg.solve_triangular(np.eye(len(be)) + L, rhs, lower=True, unit_diagonal=True)
            O = np.exp(lg)[:, None] * (Q @ S) + np.tril(D * (Q @ K.T)) @ U
            np.testing.assert_allclose(o[0, h, sl], O, rtol=1e-10, atol=1e-10)
            S = np.exp(lg[-1]) * S + (np.exp(lg[-1] - lg)[:, None] * K).T @ U
        np.testing.assert_allclose(mT[0, h], S, rtol=1e-10, atol=1e-10)


def test_update_is_a_gradient_step_on_the_regression_loss():
    # DeltaNet row with a_s = b_s = eta: M_s = M_{s-1} - eta grad_M l(M_{s-1}), l(M) = |k M - v|^2 / 2
    rng = np.random.default_rng(8)
    dk, dv, eta = 4, 3, 0.37
    M0 = rng.standard_normal((dk, dv))
    k, v = rng.standard_normal(dk), rng.standard_normal(dv)
    loss = lambda M: 0.5 * np.sum((k @ M - v) ** 2)
    grad = np.zeros_like(M0)
    h = 1e-6
    for i in range(dk):
        for j in range(dv):
            E = np.zeros_like(M0)
            E[i, j] = h
            grad[i, j] = (loss(M0 + E) - loss(M0 - E)) / (2 * h)
    eta_a = np.full((1, 1, 1), eta)
    _, mT = delta_oracle_fwd(k[None, None, None], k[None, None, None], v[None, None, None], None, eta_a, eta_a, M0[None, None])
    np.testing.assert_allclose(mT[0, 0], M0 - eta * grad, rtol=1e-8, atol=1e-8)


def test_gated_row_erases_along_the_key_and_decays_across_it():
    # Gated DeltaNet row (beta = 1) with a unit key: k_s M_s = b_s v_s, and for p orthogonal to k_s: p M_s = a_s p M_{s-1}
    rng = np.random.default_rng(9)
    dk, dv = 5, 4
    k = rng.standard_normal(dk)
    k /= np.linalg.norm(k)
    p = rng.standard_normal(dk)
    p -= (p @ k) * k
    v, M0 = rng.standard_normal(dv), rng.standard_normal((dk, dv))
    la, bb = np.full((1, 1, 1), -0.3), np.full((1, 1, 1), 0.8)
    qq = np.stack([k, p])                                   # two read-outs of the same one-token state
    for qi, want in ((k, 0.8 * v), (p, np.exp(-0.3) * (p @ M0))):
        o, _ = delta_oracle_fwd(qi[None, None, None], k[None, None, None], v[None, None, None], la, None, bb, M0[None, None])
        np.testing.assert_allclose(o[0, 0, 0], want, rtol=1e-12, atol=1e-12)
    assert qq.shape == (2, dk)


def loss_of(q, k, v, la, beta, b, M0, d_o, d_mT):
    o, mT = delta_oracle_fwd(q, k, v, la, beta, b, M0)
    return float((o * d_o).sum() + (mT * d_mT).sum())


@pytest.mark.parametrize("gated", [False, True])
def test_backward_matches_central_finite_differences(gated):
    q, k, v, la, beta, b, M0 = rand_case(B=1, H=2, T=70, dk=4, dv=3, seed=10, gated=gated, unit_keys=False)
    k *= 0.7
    rng = np.random.default_rng(11)
    d_o, d_mT = rng.standard_normal(v.shape), rng.standard_normal(M0.shape)
    r = delta_oracle_bwd(q, k, v, d_o, la, beta, b, M0, d_mT)
    args = dict(q=q, k=k, v=v, la=la, beta=beta, b=b, M0=M0)
    names = dict(q="dq", k="dk", v="dv", la="d_log_alpha", beta="d_beta", b="d_b", M0="d_m0")
    h = 1e-6
    for name, arr in args.items():
        if arr is None:
            assert r[names[name]] is None
            continue
        flat_idx = rng.choice(arr.size, size=min(arr.size, 25), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            plus, minus = dict(args), dict(args)
            plus[name] = arr.copy()
            plus[name][idx] += h
            minus[name] = arr.copy()
            minus[name][idx] -= h
            fd = (loss_of(d_o=d_o, d_mT=d_mT, **plus) - loss_of(d_o=d_o, d_mT=d_mT, **minus)) / (2 * h)
            got = r[names[name]][idx]
            assert abs(got - fd) <= 1e-6 * max(1.0, abs(fd)), (name, idx, got, fd)


def test_backward_is_linear_in_the_cotangents_and_pairs_are_independent():
    q, k, v, la, beta, b, M0 = rand_case(seed=12)
    rng = np.random.default_rng(13)
    d1, d2 = rng.standard_normal(v.shape), rng.standard_normal(v.shape)
    r1 = delta_oracle_bwd(q, k, v, d1, la, beta, b, M0)
    r2 = delta_oracle_bwd(q, k, v, d2, la, beta, b, M0)
    r12 = delta_oracle_bwd(q, k, v, 2.0 * d1 - 3.0 * d2, la, beta, b, M0)
    for n in r1:
        np.testing.assert_allclose(r12[n], 2.0 * r1[n] - 3.0 * r2[n], rtol=1e-10, atol=1e-10)
    # one (b,h) pair alone gives the same numbers as inside the batch
    one = delta_oracle_bwd(q[1:, :1], k[1:, :1], v[1:, :1], d1[1:, :1], la[1:, :1], beta[1:, :1], b[1:, :1], M0[1:, :1])
    for n in r1:
        np.testing.assert_array_equal(one[n], r1[n][1:, :1])


def test_missing_parameters_mean_one_and_empty_sequences_pass_the_state_through():
    q, k, v, la, beta, b, M0 = rand_case(seed=14)
    one = np.ones_like(beta)
    o1, m1 = delta_oracle_fwd(q, k, v, None, None, None, M0)
    o2, m2 = delta_oracle_fwd(q, k, v, np.zeros_like(beta), one, one, M0)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(m1, m2)
    o, mT = delta_oracle_fwd(q[:, :, :0], k[:, :, :0], v[:, :, :0], None, None, None, M0)
    assert o.shape[2] == 0
    np.testing.assert_array_equal(mT, M0)
