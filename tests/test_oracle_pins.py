"""Pins of the CPU oracles against what the paper and the mathematics fix.

The paper prints no numeric value of any state or output, so the oracle is
pinned by its identities instead: each test below states the passage it uses.
None of them calls the GPU library.  Tolerances are fp64 round-off levels.
"""
import json
import os

import numpy as np
import pytest

from oracle import chunk_oracle, token_oracle

RNG = np.random.default_rng


def _rand_problem(rng, T, H, dk, dv, N=1, h0=True):
    q = rng.standard_normal((N, T, H, dk)).astype(np.float32)
    k = rng.standard_normal((N, T, H, dk)).astype(np.float32)
    v = rng.standard_normal((N, T, H, dv)).astype(np.float32)
    la = -np.log1p(np.exp(rng.standard_normal((N, T, H))))
    eta = 1.0 / (1.0 + np.exp(-rng.standard_normal((N, T, H))))
    S0 = rng.standard_normal((N, H, dk, dv)) if h0 else None
    return q, k, v, la, eta, S0


def _steps(q, k, v, la, eta, eps, S0):
    """Drive the oracle one token at a time so every intermediate state is visible."""
    T = q.shape[0]
    S = S0.copy()
    states, outs = [S.copy()], []
    for t in range(T):
        o, S = token_oracle.kla_decode(q[t][None, None], k[t][None, None], v[t][None, None],
                                       np.array([[la[t]]]), np.array([[eta[t]]]), eps, S[None, None])
        S = S[0, 0]
        states.append(S.copy())
        outs.append(o[0, 0])
    return states, np.array(outs)


def test_hand_worked_example():
    """tests/golden/hand_worked_3step.json: three tokens worked by hand from Algorithm 1 (left)."""
    with open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked_3step.json")) as f:
        g = json.load(f)
    q = np.array(g["q"], np.float32)[None, :, None, :]
    k = np.array(g["k"], np.float32)[None, :, None, :]
    v = np.array(g["v"], np.float32)[None, :, None, :]
    la = np.log(np.array(g["alpha"]))[None, :, None]
    eta = np.array(g["eta"])[None, :, None]
    o, hT, _ = token_oracle.kla_recurrent(q, k, v, la, eta, g["eps"])
    np.testing.assert_allclose(o[0, :, 0, :], np.array(g["o"]), rtol=0, atol=1e-15)
    np.testing.assert_allclose(hT[0, 0], np.array(g["S_final"]), rtol=0, atol=1e-15)
    # the chunkwise route must give the same numbers (any chunk length)
    for C in (1, 2, 3):
        oc, hc = chunk_oracle.kla_chunkwise(q, k, v, la, eta, g["eps"], chunk=C)
        np.testing.assert_allclose(oc[0, :, 0, :], np.array(g["o"]), rtol=0, atol=1e-14)
        np.testing.assert_allclose(hc[0, 0], np.array(g["S_final"]), rtol=0, atol=1e-14)


def test_projection_property_theorem1():
    """Theorem 1: alpha=1, eta=1, eps=0  =>  S_t^T k_t = v_t after every write (any S_0)."""
    rng = RNG(1)
    T, dk, dv = 40, 16, 12
    q, k, v, la, eta, S0 = _rand_problem(rng, T, 1, dk, dv)
    q, k, v = q[0, :, 0], k[0, :, 0], v[0, :, 0]
    states, _ = _steps(q, k, v, np.zeros(T), np.ones(T), 0.0, S0[0, 0])
    for t in range(T):
        S = states[t + 1]
        assert np.max(np.abs(S.T @ k[t].astype(np.float64) - v[t])) <= 1e-12 * np.max(np.abs(v))


def test_residual_contraction_prop2_all_parameters():
    """Proposition 2 / eq. (9): v - S_t^T k = (1 - eta |k|^2/(|k|^2+eps)) (v - alpha S_{t-1}^T k).

    Holds for every alpha, eta, eps: pins decay-before-residual, beta and the write direction."""
    rng = RNG(2)
    T, dk, dv = 50, 8, 5
    for eps in (0.0, 1e-6, 0.3):
        q, k, v, la, eta, S0 = _rand_problem(rng, T, 1, dk, dv)
        q, k, v, la, eta = q[0, :, 0], k[0, :, 0], v[0, :, 0], la[0, :, 0], eta[0, :, 0]
        states, _ = _steps(q, k, v, la, eta, eps, S0[0, 0])
        for t in range(T):
            kk = k[t].astype(np.float64)
            nk = kk @ kk
            e_before = v[t] - np.exp(la[t]) * (states[t].T @ kk)
            e_after = v[t] - states[t + 1].T @ kk
            factor = 1.0 - eta[t] * nk / (nk + eps)
            np.testing.assert_allclose(e_after, factor * e_before, rtol=1e-11, atol=1e-12)


def test_minimum_norm_change_theorem1_i():
    """Theorem 1(i): eta=1, eps=0 => |S_t - S~|_F = |e|/|k| and <S_t - S~, H>_F = 0 whenever H^T k = 0."""
    rng = RNG(3)
    dk, dv = 10, 7
    q, k, v, la, eta, S0 = _rand_problem(rng, 1, 1, dk, dv)
    kk = k[0, 0, 0].astype(np.float64)
    alpha = np.exp(la[0, 0, 0])
    states, _ = _steps(q[0, :, 0], k[0, :, 0], v[0, :, 0], la[0, :, 0], np.ones(1), 0.0, S0[0, 0])
    S_tilde = alpha * states[0]
    delta = states[1] - S_tilde
    e = v[0, 0, 0] - S_tilde.T @ kk
    np.testing.assert_allclose(np.linalg.norm(delta), np.linalg.norm(e) / np.linalg.norm(kk), rtol=1e-12)
    for _ in range(5):
        Hm = rng.standard_normal((dk, dv))
        Hm -= np.outer(kk, kk @ Hm) / (kk @ kk)          # now H^T k = 0
        assert abs(np.sum(delta * Hm)) <= 1e-12 * np.linalg.norm(delta) * np.linalg.norm(Hm)


def test_line_search_eq4():
    """eq. (4): along S~ + tau k e^T the loss is (1/2)(1 - tau |k|^2)^2 |e|^2.  With eps=0 the
    oracle's step is tau = eta/|k|^2, so eta sweeps the path; the minimum sits at eta = 1."""
    rng = RNG(4)
    dk, dv = 6, 4
    q, k, v, la, _, S0 = _rand_problem(rng, 1, 1, dk, dv)
    kk = k[0, 0, 0].astype(np.float64)
    vv = v[0, 0, 0].astype(np.float64)
    S_tilde = np.exp(la[0, 0, 0]) * S0[0, 0]
    e = vv - S_tilde.T @ kk
    losses = []
    for eta in (0.0, 0.25, 0.9, 1.0, 1.1, 1.7):
        states, _ = _steps(q[0, :, 0], k[0, :, 0], v[0, :, 0], la[0, :, 0], np.array([eta]), 0.0, S0[0, 0])
        loss = 0.5 * np.sum((states[1].T @ kk - vv) ** 2)
        np.testing.assert_allclose(loss, 0.5 * (1.0 - eta) ** 2 * (e @ e), rtol=1e-10, atol=1e-24)
        losses.append(loss)
    assert int(np.argmin(losses)) == 3


def test_proximal_stationarity_prop1():
    """Proposition 1: S_t - S~ + mu k (S_t^T k - v)^T = 0 with mu = eta/((1-eta)|k|^2 + eps)."""
    rng = RNG(5)
    dk, dv = 9, 6
    for eta, eps in ((0.3, 0.0), (0.8, 1e-6), (1.0, 0.2), (0.5, 0.7)):
        q, k, v, la, _, S0 = _rand_problem(rng, 1, 1, dk, dv)
        kk = k[0, 0, 0].astype(np.float64)
        vv = v[0, 0, 0].astype(np.float64)
        states, _ = _steps(q[0, :, 0], k[0, :, 0], v[0, :, 0], la[0, :, 0], np.array([eta]), eps, S0[0, 0])
        S_tilde = np.exp(la[0, 0, 0]) * states[0]
        mu = eta / ((1.0 - eta) * (kk @ kk) + eps)
        grad = states[1] - S_tilde + mu * np.outer(kk, states[1].T @ kk - vv)
        assert np.max(np.abs(grad)) <= 1e-11 * max(1.0, np.max(np.abs(states[1])) * mu)


def test_pure_decay_eta_zero():
    """eq. (3) with eta=0: beta=0, so S_t = (prod alpha) S_0 and o_t = (prod alpha) S_0^T q_t."""
    rng = RNG(6)
    T, H, dk, dv = 37, 2, 8, 6
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv, N=2)
    o, hT, _ = token_oracle.kla_recurrent(q, k, v, la, np.zeros_like(eta), 1e-6, h0=S0)
    cum = np.exp(np.cumsum(la, axis=1))                       # [N,T,H]
    expect_o = cum[..., None] * np.einsum("nhkv,nthk->nthv", S0, q.astype(np.float64))
    np.testing.assert_allclose(o, expect_o, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(hT, cum[:, -1][..., None, None] * S0, rtol=1e-11, atol=1e-14)
    oc, hc = chunk_oracle.kla_chunkwise(q, k, v, la, np.zeros_like(eta), 1e-6, h0=S0, chunk=8)
    np.testing.assert_allclose(oc, expect_o, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(hc, hT, rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("C", [1, 16, 64, 150])
@pytest.mark.parametrize("with_h0", [False, True])
def test_chunkwise_equals_recurrent_props3_4(C, with_h0):
    """Propositions 3-4 (eqs. (6)-(8)): the chunkwise solver reproduces the token loop for any C,
    including T not a multiple of C, C=1 (no off-diagonal terms) and C>=T (one chunk)."""
    rng = RNG(7 + C)
    T, H, dk, dv = 150, 2, 12, 20
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv, N=2, h0=with_h0)
    la = la * 0.3                                             # slower decay: early tokens still matter at T
    o, hT, _ = token_oracle.kla_recurrent(q, k, v, la, eta, 1e-6, h0=S0)
    oc, hc = chunk_oracle.kla_chunkwise(q, k, v, la, eta, 1e-6, h0=S0, chunk=C)
    assert token_oracle.rel_err(oc, o) <= 1e-10
    assert token_oracle.rel_err(hc, hT) <= 1e-10


def test_chunk_intermediates_wy_factors():
    """Propositions 5-6 and eq. (15): U = U0 - W S_0 with W = T B D_gamma K, U0 = T B V, and the
    chunk transition P_C = gamma_C I - sum_r (gamma_C/gamma_r) k_r w_r^T equals the explicit product
    of alpha_r (I - beta_r k_r k_r^T)."""
    rng = RNG(8)
    T, dk, dv = 16, 6, 5
    q, k, v, la, eta, S0 = _rand_problem(rng, T, 1, dk, dv)
    q, k, v, la, eta = q[0, :, 0], k[0, :, 0], v[0, :, 0], la[0, :, 0], eta[0, :, 0]
    _, _, inter = chunk_oracle.kla_chunkwise_unit(q, k, v, la, eta, 1e-6, S0[0, 0], chunk=T, want=True)
    c = inter[0]
    np.testing.assert_allclose(c["U"], c["U0"] - c["W"] @ S0[0, 0], rtol=1e-11, atol=1e-12)
    kk = k.astype(np.float64)
    Pexp = np.eye(dk)
    for r in range(T):
        Pexp = np.exp(la[r]) * (np.eye(dk) - c["beta"][r] * np.outer(kk[r], kk[r])) @ Pexp
    g = c["g"]
    Pwy = np.exp(g[-1]) * np.eye(dk) - sum(np.exp(g[-1] - g[r]) * np.outer(kk[r], c["W"][r]) for r in range(T))
    np.testing.assert_allclose(Pwy, Pexp, rtol=1e-10, atol=1e-12)


def test_gdn_reduction_unit_keys():
    """Sec. 3.1 'Connection to GDN' / Table 2: with |k|=1 and eps=0 the coefficient is beta=eta and
    the update is S_t = (I - eta k k^T) alpha S_{t-1} + eta k v^T, coded here in that product form."""
    rng = RNG(9)
    T, dk, dv = 30, 8, 8
    q, k, v, la, eta, S0 = _rand_problem(rng, T, 1, dk, dv)
    k64 = k.astype(np.float64)
    k64 /= np.linalg.norm(k64, axis=-1, keepdims=True)
    k32 = k64.astype(np.float32)                              # unit norm only up to fp32 rounding
    o, hT, _ = token_oracle.kla_recurrent(q, k32, v, la, eta, 0.0, h0=S0)
    S = S0[0, 0].copy()
    for t in range(T):
        kk = k32[0, t, 0].astype(np.float64)
        b = eta[0, t, 0] / (kk @ kk)                          # = eta up to 1e-7
        assert abs(b - eta[0, t, 0]) < 1e-6
        S = (np.eye(dk) - eta[0, t, 0] * np.outer(kk, kk)) @ (np.exp(la[0, t, 0]) * S) \
            + eta[0, t, 0] * np.outer(kk, v[0, t, 0])
        np.testing.assert_allclose(o[0, t, 0], S.T @ q[0, t, 0], rtol=0, atol=2e-6 * (1 + np.max(np.abs(S))))
    np.testing.assert_allclose(hT[0, 0], S, rtol=0, atol=2e-6 * (1 + np.max(np.abs(S))))


def test_bruteforce_product_form_table5():
    """Table 5 (KLA row): o_t = sum_{j<=t} beta_j v_j k_j^T [M_{j+1} ... M_t] q_t with
    M_s = alpha_s (I - beta_s k_s k_s^T), the factor s=j+1 next to k_j; S_0 = 0; tiny sizes."""
    rng = RNG(10)
    T, dk, dv = 7, 4, 3
    q, k, v, la, eta, _ = _rand_problem(rng, T, 1, dk, dv, h0=False)
    eps = 1e-3
    o, _, _ = token_oracle.kla_recurrent(q, k, v, la, eta, eps)
    kk, vv, qq = k[0, :, 0].astype(np.float64), v[0, :, 0].astype(np.float64), q[0, :, 0].astype(np.float64)
    beta = eta[0, :, 0] / (np.sum(kk * kk, axis=1) + eps)
    M = [np.exp(la[0, s, 0]) * (np.eye(dk) - beta[s] * np.outer(kk[s], kk[s])) for s in range(T)]
    for t in range(T):
        acc = np.zeros(dv)
        for j in range(t + 1):
            prod = np.eye(dk)
            for s in range(j + 1, t + 1):
                prod = prod @ M[s]
            acc += beta[j] * vv[j] * (kk[j] @ prod @ qq[t])
        np.testing.assert_allclose(o[0, t, 0], acc, rtol=1e-10, atol=1e-12)


def test_textbook_kaczmarz_limits():
    """Sec. 3.1 (row-action method): alpha=1, eta=1, eps=0, S_0=0.
    (a) orthonormal keys: one pass gives S = sum_i k_i v_i^T exactly;
    (b) T<=d_k independent keys swept cyclically converge to the minimum-norm solution pinv(K) V."""
    rng = RNG(11)
    dk, dv, T = 12, 5, 6
    Qm, _ = np.linalg.qr(rng.standard_normal((dk, dk)))
    K = Qm[:, :T].T.astype(np.float32)                         # rows orthonormal up to fp32 rounding
    V = rng.standard_normal((T, dv)).astype(np.float32)
    ones, zeros = np.ones((1, T, 1)), np.zeros((1, T, 1))
    _, hT, _ = token_oracle.kla_recurrent(K[None, :, None], K[None, :, None], V[None, :, None], zeros, ones, 0.0)
    np.testing.assert_allclose(hT[0, 0], K.astype(np.float64).T @ V, rtol=0, atol=5e-6)
    K = rng.standard_normal((T, dk)).astype(np.float32)
    sweeps = 400
    Kc, Vc = np.tile(K, (sweeps, 1)), np.tile(V, (sweeps, 1))
    n = T * sweeps
    _, hT, _ = token_oracle.kla_recurrent(Kc[None, :, None], Kc[None, :, None], Vc[None, :, None],
                                          np.zeros((1, n, 1)), np.ones((1, n, 1)), 0.0)
    np.testing.assert_allclose(hT[0, 0], np.linalg.pinv(K.astype(np.float64)) @ V, rtol=0, atol=1e-9)


def test_scaling_metamorphic_and_zero_key():
    """eps=0: (k, q) -> (c k, c q) leaves every o_t unchanged and scales h_T by 1/c (beta ~ 1/c^2).
    A zero key with eps=0 must write nothing and give finite numbers (beta := 0 reading)."""
    rng = RNG(12)
    T, dk, dv = 25, 8, 8
    q, k, v, la, eta, _ = _rand_problem(rng, T, 1, dk, dv, h0=False)
    o1, h1, _ = token_oracle.kla_recurrent(q, k, v, la, eta, 0.0)
    o2, h2, _ = token_oracle.kla_recurrent(4 * q, 4 * k, v, la, eta, 0.0)
    np.testing.assert_allclose(o2, o1, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(h2, h1 / 4, rtol=1e-12, atol=1e-14)
    k[0, 5, 0] = 0.0
    o3, h3, _ = token_oracle.kla_recurrent(q, k, v, la, eta, 0.0)
    assert np.all(np.isfinite(o3)) and np.all(np.isfinite(h3))
    oc, hc = chunk_oracle.kla_chunkwise(q, k, v, la, eta, 0.0, chunk=8)
    assert token_oracle.rel_err(oc, o3) <= 1e-10 and token_oracle.rel_err(hc, h3) <= 1e-10


def test_batch_head_independence_and_varlen():
    """Every (sequence, head) is an independent recurrence (Algorithm 1 is per head): permuting
    heads permutes outputs; a packed batch equals the sequences run one by one."""
    rng = RNG(13)
    T, H, dk, dv = 50, 3, 6, 4
    q, k, v, la, eta, _ = _rand_problem(rng, T, H, dk, dv, h0=False)
    o, hT, _ = token_oracle.kla_recurrent(q, k, v, la, eta, 1e-6)
    perm = [2, 0, 1]
    op, hp, _ = token_oracle.kla_recurrent(q[:, :, perm], k[:, :, perm], v[:, :, perm], la[:, :, perm],
                                           eta[:, :, perm], 1e-6)
    np.testing.assert_array_equal(op, o[:, :, perm])
    np.testing.assert_array_equal(hp, hT[:, perm])
    cu = [0, 13, 30, 50]
    h0 = rng.standard_normal((3, H, dk, dv))
    ov, hv, _ = token_oracle.kla_recurrent(q, k, v, la, eta, 1e-6, h0=h0, cu_seqlens=cu)
    for s in range(3):
        a, b = cu[s], cu[s + 1]
        os_, hs, _ = token_oracle.kla_recurrent(q[:, a:b], k[:, a:b], v[:, a:b], la[:, a:b], eta[:, a:b],
                                                1e-6, h0=h0[s:s + 1])
        np.testing.assert_array_equal(ov[:, a:b], os_)
        np.testing.assert_array_equal(hv[s], hs[0])
    oc, hc = chunk_oracle.kla_chunkwise(q, k, v, la, eta, 1e-6, h0=h0, cu_seqlens=cu, chunk=16)
    assert token_oracle.rel_err(oc, ov) <= 1e-10 and token_oracle.rel_err(hc, hv) <= 1e-10


def test_split_invariance():
    """The state is the only carry (Sec. 2): running T1 tokens, then T2 from h_T, equals one run."""
    rng = RNG(14)
    T, H, dk, dv = 60, 2, 8, 8
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv)
    o, hT, _ = token_oracle.kla_recurrent(q, k, v, la, eta, 1e-6, h0=S0)
    a = 23
    o1, h1, _ = token_oracle.kla_recurrent(q[:, :a], k[:, :a], v[:, :a], la[:, :a], eta[:, :a], 1e-6, h0=S0)
    o2, h2, _ = token_oracle.kla_recurrent(q[:, a:], k[:, a:], v[:, a:], la[:, a:], eta[:, a:], 1e-6, h0=h1)
    np.testing.assert_array_equal(np.concatenate([o1, o2], axis=1), o)
    np.testing.assert_array_equal(h2, hT)


def test_option_gdn_beta_product_form():
    """Option gdn_beta (beta_t = eta_t, Table 2's gated delta rule) against the product form
    S_t = (I - eta k k^T) alpha S_{t-1} + eta k v^T for keys of ANY norm, and against the default
    coefficient after the substitution eta -> eta (|k|^2 + eps) that makes the two rules coincide."""
    rng = RNG(21)
    T, dk, dv = 25, 6, 5
    q, k, v, la, eta, S0 = _rand_problem(rng, T, 1, dk, dv)
    k *= 0.3                                                  # keep I - eta k k^T a contraction
    eps = 1e-3
    o, hT, _ = token_oracle.kla_recurrent(q, k, v, la, eta, eps, h0=S0, gdn_beta=True)
    S = S0[0, 0].copy()
    for t in range(T):
        kk = k[0, t, 0].astype(np.float64)
        S = (np.eye(dk) - eta[0, t, 0] * np.outer(kk, kk)) @ (np.exp(la[0, t, 0]) * S) \
            + eta[0, t, 0] * np.outer(kk, v[0, t, 0])
        np.testing.assert_allclose(o[0, t, 0], S.T @ q[0, t, 0], rtol=0, atol=1e-12 * (1 + np.max(np.abs(S))))
    np.testing.assert_allclose(hT[0, 0], S, rtol=0, atol=1e-12 * (1 + np.max(np.abs(S))))
    nk = np.sum(k.astype(np.float64) ** 2, axis=-1)
    o2, hT2, _ = token_oracle.kla_recurrent(q, k, v, la, eta * (nk + eps), eps, h0=S0)
    np.testing.assert_allclose(o2, o, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(hT2, hT, rtol=1e-12, atol=1e-13)
    # and it is not the default rule
    o3, _, _ = token_oracle.kla_recurrent(q, k, v, la, eta, eps, h0=S0)
    assert np.max(np.abs(o3 - o)) > 1e-3


def test_option_normalize_q():
    """Option normalize_q (Sec. 3.3: o_t = S_t^T q_t / |q_t|): equals the plain readout divided by numpy's
    norm, does not depend on the scale of q, leaves the states alone, and gives 0 for a zero query."""
    rng = RNG(22)
    T, H, dk, dv = 12, 2, 5, 4
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv)
    q[0, 3, 1] = 0.0
    eps = 1e-6
    o, hT, _ = token_oracle.kla_recurrent(q, k, v, la, eta, eps, h0=S0)
    on, hTn, _ = token_oracle.kla_recurrent(q, k, v, la, eta, eps, h0=S0, normalize_q=True)
    nq = np.linalg.norm(q.astype(np.float64), axis=-1, keepdims=True)
    want = np.divide(o, nq, out=np.zeros_like(o), where=nq > 0)
    np.testing.assert_allclose(on, want, rtol=1e-13, atol=0)
    assert np.all(on[0, 3, 1] == 0.0)
    np.testing.assert_array_equal(hTn, hT)
    scale = np.exp2(rng.integers(-3, 4, size=(1, T, H, 1))).astype(np.float32)   # exact in fp32
    os_, _, _ = token_oracle.kla_recurrent(q * scale, k, v, la, eta, eps, h0=S0, normalize_q=True)
    np.testing.assert_allclose(os_, on, rtol=1e-13, atol=0)
    # decode entry point takes the same options
    od, Sd = token_oracle.kla_decode(q[:, 0], k[:, 0], v[:, 0], la[:, 0], eta[:, 0], eps, S0, normalize_q=True, gdn_beta=True)
    og, hg, _ = token_oracle.kla_recurrent(q[:, :1], k[:, :1], v[:, :1], la[:, :1], eta[:, :1], eps, h0=S0,
                                           normalize_q=True, gdn_beta=True)
    np.testing.assert_allclose(od, og[:, 0], rtol=1e-14, atol=0)
    np.testing.assert_allclose(Sd, hg, rtol=1e-14, atol=0)


# ---- gradient oracle (reverse accumulation through Algorithm 1, left panel) ----------------------
def _loss(q, k, v, la, eta, eps, S0, go, ghT):
    o, hT, _ = token_oracle.kla_recurrent(q, k, v, la, eta, eps, h0=S0, threads=1)
    return float(np.sum(o * go) + np.sum(hT * ghT))


def test_gradient_central_differences():
    """The gradient oracle against central finite differences of the (separately pinned) forward oracle.

    q, k, v sit on a 2^-6 grid and move by 2^-9, so the perturbed fp32 inputs are exact; the sequence spans two
    of the gradient oracle's 64-token checkpoint segments plus a ragged tail, with non-zero h0 and d_hT."""
    rng = RNG(41)
    T, H, dk, dv, eps = 133, 2, 4, 3, 1e-3
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv)
    q, k, v = (np.round(x * 64) / 64 for x in (q, k, v))
    q, k, v = q.astype(np.float32), k.astype(np.float32), v.astype(np.float32)
    la = la * 0.2                                             # slow decay: early tokens still reach the loss
    go = rng.standard_normal((1, T, H, dv))
    ghT = rng.standard_normal((1, H, dk, dv))
    g = token_oracle.kla_recurrent_bwd(q, k, v, la, eta, eps, go, h0=S0, d_hT=ghT)
    args = {"q": q, "k": k, "v": v, "la": la, "eta": eta, "S0": S0}
    names = {"q": "dq", "k": "dk", "v": "dv", "la": "dlog_alpha", "eta": "deta", "S0": "dh0"}
    for name, arr in args.items():
        h = 2.0 ** -9 if arr.dtype == np.float32 else 1e-5
        flat_idx = rng.choice(arr.size, size=10, replace=False)
        flat_idx[0] = 0                                       # always include the first token
        scale = np.max(np.abs(g[names[name]]))
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            plus, minus = arr.copy(), arr.copy()
            plus[idx] += h
            minus[idx] -= h
            a_p = dict(args); a_p[name] = plus
            a_m = dict(args); a_m[name] = minus
            fd = (_loss(a_p["q"], a_p["k"], a_p["v"], a_p["la"], a_p["eta"], eps, a_p["S0"], go, ghT)
                  - _loss(a_m["q"], a_m["k"], a_m["v"], a_m["la"], a_m["eta"], eps, a_m["S0"], go, ghT)) / (2 * h)
            assert abs(fd - g[names[name]][idx]) <= 2e-5 * scale + 1e-8, (name, idx, fd, g[names[name]][idx])


def test_gradient_single_step_closed_form():
    """One token: o = S_1^T q with S_1 = alpha (I - beta k k^T) h0 + beta k v^T (eq. (5) transposed), so
    L = q^T S_1 d_o is an explicit polynomial in the inputs; its partial derivatives are written out here."""
    rng = RNG(42)
    dk, dv, eps = 5, 4, 0.37
    q, k, v, la, eta, S0 = _rand_problem(rng, 1, 1, dk, dv)
    go = rng.standard_normal((1, 1, 1, dv))
    g = token_oracle.kla_recurrent_bwd(q, k, v, la, eta, eps, go, h0=S0)
    qq, kk, vv, d = (x[0, 0, 0].astype(np.float64) for x in (q, k, v, go))
    al, et, h0 = float(np.exp(la[0, 0, 0])), float(eta[0, 0, 0]), S0[0, 0]
    den = kk @ kk + eps
    beta = et / den
    qk, hd = qq @ kk, h0 @ d                                  # h0 d is a d_k vector
    # L = alpha q.(h0 d) - alpha beta (q.k)(k.(h0 d)) + beta (q.k)(v.d)
    bracket = -al * qk * (kk @ hd) + qk * (vv @ d)            # dL/dbeta
    S1 = al * (h0 - beta * np.outer(kk, kk @ h0)) + beta * np.outer(kk, vv)
    np.testing.assert_allclose(g["dq"][0, 0, 0], S1 @ d, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dv"][0, 0, 0], beta * qk * d, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["deta"][0, 0, 0], bracket / den, rtol=1e-12)
    np.testing.assert_allclose(g["dlog_alpha"][0, 0, 0], al * (qq @ hd - beta * qk * (kk @ hd)), rtol=1e-12)
    dk_expect = (-al * beta * (qq * (kk @ hd) + qk * hd) + beta * qq * (vv @ d)
                 - 2.0 * beta / den * bracket * kk)
    np.testing.assert_allclose(g["dk"][0, 0, 0], dk_expect, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g["dh0"][0, 0], al * (np.outer(qq, d) - beta * qk * np.outer(kk, d)), rtol=1e-12, atol=1e-14)


def test_gradient_eta_zero_closed_form():
    """eta = 0: S_t = Gamma_t h0 (Gamma_t the decay product), so dq_t = Gamma_t h0 d_o_t, dh0 = sum_t Gamma_t q_t d_o_t^T
    + Gamma_T d_hT, dlog_alpha_r = sum_{t>=r} Gamma_t q_t^T h0 d_o_t + Gamma_T <d_hT, h0>, and dk = dv = 0 because
    the write vanishes together with the derivative of beta with respect to k."""
    rng = RNG(43)
    T, H, dk, dv = 90, 2, 6, 5
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv, N=2)
    go = rng.standard_normal((2, T, H, dv))
    ghT = rng.standard_normal((2, H, dk, dv))
    g = token_oracle.kla_recurrent_bwd(q, k, v, la, np.zeros_like(eta), 1e-6, go, h0=S0, d_hT=ghT)
    cum = np.exp(np.cumsum(la, axis=1))
    q64 = q.astype(np.float64)
    np.testing.assert_allclose(g["dq"], cum[..., None] * np.einsum("nhkv,nthv->nthk", S0, go), rtol=1e-10, atol=1e-12)
    dh0 = np.einsum("nth,nthk,nthv->nhkv", cum, q64, go) + cum[:, -1][..., None, None] * ghT
    np.testing.assert_allclose(g["dh0"], dh0, rtol=1e-10, atol=1e-12)
    per_t = cum * np.einsum("nthk,nhkv,nthv->nth", q64, S0, go)
    tail = np.flip(np.cumsum(np.flip(per_t, axis=1), axis=1), axis=1)
    dla = tail + (cum[:, -1] * np.einsum("nhkv,nhkv->nh", ghT, S0))[:, None, :]
    np.testing.assert_allclose(g["dlog_alpha"], dla, rtol=1e-9, atol=1e-11)
    assert np.max(np.abs(g["dk"])) == 0.0 and np.max(np.abs(g["dv"])) == 0.0
    assert np.max(np.abs(g["deta"])) > 0.0                    # d beta / d eta = 1/(||k||^2+eps) is not zero


def test_gradient_packed_equals_separate():
    """Sequences of a packed batch are independent: gradients equal those of each sequence run alone."""
    rng = RNG(44)
    lens = [70, 1, 129]
    cu = np.concatenate([[0], np.cumsum(lens)])
    T, H, dk, dv = int(cu[-1]), 2, 4, 4
    q, k, v, la, eta, _ = _rand_problem(rng, T, H, dk, dv, h0=False)
    S0 = rng.standard_normal((3, H, dk, dv))
    go = rng.standard_normal((1, T, H, dv))
    ghT = rng.standard_normal((3, H, dk, dv))
    g = token_oracle.kla_recurrent_bwd(q, k, v, la, eta, 1e-4, go, h0=S0, d_hT=ghT, cu_seqlens=cu)
    for s in range(3):
        a, b = int(cu[s]), int(cu[s + 1])
        gs = token_oracle.kla_recurrent_bwd(q[:, a:b], k[:, a:b], v[:, a:b], la[:, a:b], eta[:, a:b], 1e-4, go[:, a:b],
                                            h0=S0[s:s + 1], d_hT=ghT[s:s + 1])
        for name in ("dq", "dk", "dv", "dlog_alpha", "deta"):
            np.testing.assert_array_equal(g[name][:, a:b], gs[name])
        np.testing.assert_array_equal(g["dh0"][s], gs["dh0"][0])


@pytest.mark.parametrize("C", [1, 16, 64])
def test_chunkwise_gradient_equals_recurrent(C):
    """Eqs. (6)-(8) differentiated chunk by chunk give the gradient of the tokenwise recurrence (two independent
    routes: numpy chunk algebra vs the C reverse accumulation), for several chunk sizes and a ragged tail."""
    rng = RNG(45)
    T, H, dk, dv, eps = 150, 1, 6, 5, 1e-3
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv)
    la = la * 0.3
    go = rng.standard_normal((1, T, H, dv))
    ghT = rng.standard_normal((1, H, dk, dv))
    ref = token_oracle.kla_recurrent_bwd(q, k, v, la, eta, eps, go, h0=S0, d_hT=ghT)
    got = chunk_oracle.kla_chunkwise_bwd_unit(q[0, :, 0], k[0, :, 0], v[0, :, 0], la[0, :, 0], eta[0, :, 0], eps,
                                              go[0, :, 0], h0=S0[0, 0], d_hT=ghT[0, 0], chunk=C)
    for name in ("dq", "dk", "dv", "dlog_alpha", "deta"):
        r = ref[name][0, :, 0]
        assert np.max(np.abs(got[name] - r)) <= 1e-9 * np.max(np.abs(r)), name
    assert np.max(np.abs(got["dh0"] - ref["dh0"][0, 0])) <= 1e-9 * np.max(np.abs(ref["dh0"]))


# ---- diagonal gating (App. B, "Extension to diagonal gating") -----------------------------------------
def _rand_diag(rng, T, H, dk, dv, N=1):
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv, N=N)
    lad = -np.log1p(np.exp(rng.standard_normal((N, T, H, dk))))
    return q, k, v, lad, eta, S0


def test_diag_equal_channels_is_scalar_gating():
    """diag(alpha) with all channels equal is alpha I: the diagonal oracle then repeats the scalar one."""
    rng = RNG(51)
    T, H, dk, dv = 40, 2, 6, 5
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv, N=2)
    lad = np.repeat(la[..., None], dk, axis=-1)
    o1, h1, _ = token_oracle.kla_recurrent(q, k, v, la, eta, 1e-3, h0=S0)
    o2, h2, _ = token_oracle.kla_recurrent_diag(q, k, v, lad, eta, 1e-3, h0=S0)
    np.testing.assert_allclose(o2, o1, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(h2, h1, rtol=1e-13, atol=1e-15)


def test_diag_options_reduce_to_the_scalar_options_and_to_their_definitions():
    """The options of the diagonal-gating oracle.  With equal channels they repeat the (separately pinned) options of
    the scalar oracle; with distinct channels the normalised read-out is the plain one divided by ||q_t|| row by row
    (0 for a zero query, states untouched), and beta_t = eta_t equals the Kaczmarz coefficient fed with
    eta_t (||k_t||^2 + eps) - eq. (3) solved for eta."""
    rng = RNG(56)
    T, H, dk, dv, eps = 30, 2, 6, 5, 1e-3
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv, N=2)
    k = (k * 0.4).astype(np.float32)                          # keeps the plain delta rule stable
    q[1, 4, 0] = 0.0
    lad = np.repeat(la[..., None], dk, axis=-1)
    for nq, gdn in ((True, False), (False, True), (True, True)):
        o1, h1, _ = token_oracle.kla_recurrent(q, k, v, la, eta, eps, h0=S0, normalize_q=nq, gdn_beta=gdn)
        o2, h2, _ = token_oracle.kla_recurrent_diag(q, k, v, lad, eta, eps, h0=S0, normalize_q=nq, gdn_beta=gdn)
        np.testing.assert_allclose(o2, o1, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(h2, h1, rtol=1e-13, atol=1e-15)
    lad2 = -np.log1p(np.exp(rng.standard_normal((2, T, H, dk))))
    o0, h0_, _ = token_oracle.kla_recurrent_diag(q, k, v, lad2, eta, eps, h0=S0)
    on, hn, _ = token_oracle.kla_recurrent_diag(q, k, v, lad2, eta, eps, h0=S0, normalize_q=True)
    nq_ = np.linalg.norm(q.astype(np.float64), axis=-1, keepdims=True)
    np.testing.assert_allclose(on, np.where(nq_ == 0, 0.0, o0 / np.where(nq_ == 0, 1.0, nq_)), rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(hn, h0_)
    assert np.all(on[1, 4, 0] == 0.0)
    eta_eq = eta * (np.sum(k.astype(np.float64) ** 2, axis=-1) + eps)
    og, hg, _ = token_oracle.kla_recurrent_diag(q, k, v, lad2, eta, eps, h0=S0, gdn_beta=True)
    ok_, hk, _ = token_oracle.kla_recurrent_diag(q, k, v, lad2, eta_eq, eps, h0=S0)
    np.testing.assert_allclose(og, ok_, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(hg, hk, rtol=1e-12, atol=1e-14)
    # one decode step with the options is one token of the sequence oracle
    od, Sd = token_oracle.kla_decode_diag(q[:, 0], k[:, 0], v[:, 0], lad2[:, 0], eta[:, 0], eps, S0, normalize_q=True, gdn_beta=True)
    o1, h1, _ = token_oracle.kla_recurrent_diag(q[:, :1], k[:, :1], v[:, :1], lad2[:, :1], eta[:, :1], eps, h0=S0,
                                                normalize_q=True, gdn_beta=True)
    np.testing.assert_allclose(od, o1[:, 0], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(Sd, h1, rtol=1e-13, atol=1e-15)


def test_diag_projection_property_is_decay_agnostic():
    """App. A, decay-agnostic remark: with eta = 1, eps = 0 the written state satisfies S_t^T k_t = v_t whatever
    linear decay produced the base point; and the residual contracts by 1 - eta |k|^2/(|k|^2+eps) in general."""
    rng = RNG(52)
    T, dk, dv = 12, 7, 4
    q, k, v, lad, eta, S0 = _rand_diag(rng, T, 1, dk, dv)
    S = S0[0, 0].copy()
    for t in range(T):
        kt = k[0, t, 0].astype(np.float64)
        S_tilde = np.exp(lad[0, t, 0])[:, None] * S
        e = v[0, t, 0] - S_tilde.T @ kt
        _, S1 = token_oracle.kla_decode_diag(q[0, t][None], k[0, t][None], v[0, t][None], lad[0, t][None], np.ones((1, 1)), 0.0, S[None, None])
        assert np.max(np.abs(S1[0, 0].T @ kt - v[0, t, 0])) <= 1e-12 * np.max(np.abs(v[0, t, 0]))
        eps, et = 0.3, float(eta[0, t, 0])
        _, S2 = token_oracle.kla_decode_diag(q[0, t][None], k[0, t][None], v[0, t][None], lad[0, t][None], np.array([[et]]), eps, S[None, None])
        nk = kt @ kt
        np.testing.assert_allclose(v[0, t, 0] - S2[0, 0].T @ kt, (1.0 - et * nk / (nk + eps)) * e, rtol=1e-11, atol=1e-13)
        S = S2[0, 0]


def test_diag_product_form_brute_force():
    """S_T = M_T ... M_1 S_0 + sum_j M_T ... M_{j+1} beta_j k_j v_j^T with the explicit d_k x d_k transitions
    M_s = (I - beta_s k_s k_s^T) diag(alpha_s) (eq. (5) with the diagonal decay operator), and o_t = S_t^T q_t."""
    rng = RNG(53)
    T, dk, dv, eps = 7, 4, 3, 1e-2
    q, k, v, lad, eta, S0 = _rand_diag(rng, T, 1, dk, dv)
    o, hT, _ = token_oracle.kla_recurrent_diag(q, k, v, lad, eta, eps, h0=S0)
    S = S0[0, 0].copy()
    for t in range(T):
        kt = k[0, t, 0].astype(np.float64)
        beta = eta[0, t, 0] / (kt @ kt + eps)
        M = (np.eye(dk) - beta * np.outer(kt, kt)) @ np.diag(np.exp(lad[0, t, 0]))
        S = M @ S + beta * np.outer(kt, v[0, t, 0])
        np.testing.assert_allclose(o[0, t, 0], S.T @ q[0, t, 0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(hT[0, 0], S, rtol=1e-12, atol=1e-14)


def test_diag_pure_decay_eta_zero():
    """eta = 0: every row of the state decays by its own running product."""
    rng = RNG(54)
    T, H, dk, dv = 33, 2, 5, 4
    q, k, v, lad, eta, S0 = _rand_diag(rng, T, H, dk, dv)
    o, hT, _ = token_oracle.kla_recurrent_diag(q, k, v, lad, np.zeros_like(eta), 1e-6, h0=S0)
    cum = np.exp(np.cumsum(lad, axis=1))                                  # [N,T,H,dk]
    np.testing.assert_allclose(hT, cum[:, -1][..., None] * S0, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(o, np.einsum("nthk,nhkv,nthk->nthv", cum, S0, q.astype(np.float64)), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("C", [1, 16, 64])
def test_diag_chunkwise_equals_recurrent(C):
    """The elementwise-decay chunk algebra (App. B) against the token loop, with a ragged tail and h0."""
    rng = RNG(55)
    T, dk, dv, eps = 150, 6, 5, 1e-3
    q, k, v, lad, eta, S0 = _rand_diag(rng, T, 1, dk, dv)
    o, hT, _ = token_oracle.kla_recurrent_diag(q, k, v, lad, eta, eps, h0=S0)
    oc, hc = chunk_oracle.kla_chunkwise_diag_unit(q[0, :, 0], k[0, :, 0], v[0, :, 0], lad[0, :, 0], eta[0, :, 0], eps,
                                                  h0=S0[0, 0], chunk=C)
    assert np.max(np.abs(oc - o[0, :, 0])) <= 1e-10 * np.max(np.abs(o))
    assert np.max(np.abs(hc - hT[0, 0])) <= 1e-10 * np.max(np.abs(hT))


def test_gradient_gdn_beta_central_differences():
    """beta_t = eta_t: the gradient oracle's option against central differences of the forward oracle's option."""
    rng = RNG(46)
    T, H, dk, dv, eps = 70, 1, 4, 3, 1e-3
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv)
    q, k, v = ((np.round(x * 64) / 64).astype(np.float32) for x in (q, k, v))
    k = k * 0.5                                              # keeps eta |k|^2 below 2, so the delta rule stays stable
    la = la * 0.2
    go = rng.standard_normal((1, T, H, dv))
    g = token_oracle.kla_recurrent_bwd(q, k, v, la, eta, eps, go, h0=S0, gdn_beta=True)
    def loss(qq, kk, ee):
        o, _, _ = token_oracle.kla_recurrent(qq, kk, v, la, ee, eps, h0=S0, threads=1, gdn_beta=True)
        return float(np.sum(o * go))
    for name, arr, key in (("k", k, "dk"), ("eta", eta, "deta"), ("q", q, "dq")):
        h = 2.0 ** -9 if arr.dtype == np.float32 else 1e-5
        scale = np.max(np.abs(g[key]))
        for fi in rng.choice(arr.size, size=8, replace=False):
            idx = np.unravel_index(fi, arr.shape)
            plus, minus = arr.copy(), arr.copy()
            plus[idx] += h
            minus[idx] -= h
            args_p = dict(qq=q, kk=k, ee=eta); args_m = dict(args_p)
            args_p[{"k": "kk", "eta": "ee", "q": "qq"}[name]] = plus
            args_m[{"k": "kk", "eta": "ee", "q": "qq"}[name]] = minus
            fd = (loss(**args_p) - loss(**args_m)) / (2 * h)
            assert abs(fd - g[key][idx]) <= 2e-5 * scale + 1e-8, (name, idx, fd, g[key][idx])


def test_gradient_normalize_q_central_differences_and_scale_invariance():
    """Read-out o_t = S_t^T q_t / ||q_t|| (Sec. 3.3): the gradient oracle's option against central differences
    of the forward oracle's option; o_t does not change when q_t is scaled by c > 0, so <q_t, dq_t> = 0 (Euler);
    a zero query has o_t = 0 and takes no gradient, and the other gradients equal those of the plain read-out
    fed with d_o / ||q||."""
    rng = RNG(47)
    T, H, dk, dv, eps = 70, 2, 4, 3, 1e-3
    q, k, v, la, eta, S0 = _rand_problem(rng, T, H, dk, dv)
    q, k, v = ((np.round(x * 64) / 64).astype(np.float32) for x in (q, k, v))
    q[0, 5, 1] = 0.0
    go = rng.standard_normal((1, T, H, dv))
    ghT = rng.standard_normal((1, H, dk, dv))
    g = token_oracle.kla_recurrent_bwd(q, k, v, la, eta, eps, go, h0=S0, d_hT=ghT, normalize_q=True)
    assert np.all(g["dq"][0, 5, 1] == 0.0)
    assert np.max(np.abs(np.sum(g["dq"] * q, axis=-1))) <= 1e-12 * np.max(np.abs(g["dq"]))
    nq = np.linalg.norm(q.astype(np.float64), axis=-1, keepdims=True)
    rn = np.where(nq == 0.0, 0.0, 1.0 / np.where(nq == 0.0, 1.0, nq))
    gp = token_oracle.kla_recurrent_bwd(q, k, v, la, eta, eps, go * rn, h0=S0, d_hT=ghT)
    for key in ("dk", "dv", "dlog_alpha", "deta", "dh0"):
        assert np.max(np.abs(g[key] - gp[key])) <= 1e-12 * np.max(np.abs(gp[key])), key

    def loss(qq, kk, vv, ll, ee):
        o, hT, _ = token_oracle.kla_recurrent(qq, kk, vv, ll, ee, eps, h0=S0, threads=1, normalize_q=True)
        return float(np.sum(o * go) + np.sum(hT * ghT))
    base = dict(qq=q, kk=k, vv=v, ll=la, ee=eta)
    for name, key in (("qq", "dq"), ("kk", "dk"), ("vv", "dv"), ("ll", "dlog_alpha"), ("ee", "deta")):
        arr = base[name]
        h = 2.0 ** -9 if arr.dtype == np.float32 else 1e-5
        scale = np.max(np.abs(g[key]))
        for fi in rng.choice(arr.size, size=6, replace=False):
            idx = np.unravel_index(fi, arr.shape)
            if name == "qq" and not np.any(q[idx[:-1]]):
                continue
            plus, minus = arr.copy(), arr.copy()
            plus[idx] += h
            minus[idx] -= h
            fd = (loss(**{**base, name: plus}) - loss(**{**base, name: minus})) / (2 * h)
            assert abs(fd - g[key][idx]) <= 5e-5 * scale + 1e-8, (name, idx, fd, g[key][idx])


def test_rel_err_metric_by_hand():
    """The parity metric every GPU test rests on, max|x - ref| / max|ref| over the whole tensor, on arrays worked by hand:
    the largest deviation (0.5, at the entry whose reference is -8) over the largest reference magnitude (8); a zero
    reference falls back to the absolute deviation; empty tensors compare equal; the metric is not symmetric."""
    ref = np.array([[1.0, -8.0], [2.0, 0.0]])
    x = np.array([[1.25, -7.5], [2.0, 0.125]])
    assert token_oracle.rel_err(x, ref) == 0.5 / 8.0
    assert token_oracle.rel_err(ref, x) == 0.5 / 7.5
    assert token_oracle.rel_err(ref, ref) == 0.0
    assert token_oracle.rel_err(np.array([0.0, -0.25]), np.zeros(2)) == 0.25
    assert token_oracle.rel_err(np.zeros((0, 3)), np.zeros((0, 3))) == 0.0
    assert token_oracle.rel_err(np.array([3.0], dtype=np.float32), np.array([2.0])) == 0.5
    assert np.isnan(token_oracle.rel_err(np.array([np.nan, 1.0]), np.array([1.0, 1.0])))
