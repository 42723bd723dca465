"""fp64 numpy oracle for the chunkwise form of Kaczmarz Linear Attention.

TEST INFRASTRUCTURE ONLY (tests, smoke check, CPU-baseline leg).  Independent
of the HIP sources and of the C token oracle: it is a second route to the same
result, used to pin "chunkwise == recurrent" (Propositions 3 and 4) and to give
the per-chunk intermediates (T, P, U, chunk states, and the WY factors W, U0 of
Propositions 5 and 6) that a single GPU kernel can be compared against.

Steps and notation are those of Algorithm 1 (right panel) and eqs. (6)-(8):
    gamma_i = prod_{r<=i} alpha_r  (restarting at each chunk),  beta_i = eta_i/(||k_i||^2+eps)
    A_ij = gamma_i/gamma_j (j<=i),  A^- its strict lower part,  B = diag(beta)
    (I + B (A^- o K K^T)) U = B (V - D_gamma K S_0)                       eq. (6)
    O = D_gamma Q S_0 + (A o Q K^T) U                                       eq. (7)
    S_out = gamma_C S_0 + K^T diag(gamma_C/gamma_i) U                       eq. (8)
Readings: every ratio gamma_i/gamma_j is formed as exp(g_i - g_j) from the
chunk-local running sum g of log alpha (the quotient itself can underflow);
the appendix's inclusive product gamma_{j->i} is read as gamma_i/gamma_j, which
is what its own induction step and eqs. (6)-(8) use; the leading term of the
w-recursion (eq. (11)) is gamma_i k_i, i.e. W = T B D_gamma K, which is what makes
T B (V - D_gamma K S_0) = U0 - W S_0.  A ragged last chunk is simply shorter.
The triangular solve is scipy's; everything else is plain numpy matmuls.
"""
from __future__ import annotations

import numpy as np
from scipy.linalg import solve_triangular


def chunk_objects(k, log_alpha, eta, eps):
    """beta, g, A (lower incl. diagonal), L = B (A^- o K K^T) for one chunk (k: [c, dk])."""
    k = np.asarray(k, dtype=np.float64)
    la = np.asarray(log_alpha, dtype=np.float64)
    et = np.asarray(eta, dtype=np.float64)
    c = k.shape[0]
    nk = np.sum(k * k, axis=1)
    den = nk + eps
    beta = np.where(den == 0.0, 0.0, et / np.where(den == 0.0, 1.0, den))
    g = np.cumsum(la)
    diff = g[:, None] - g[None, :]
    lower = np.tril(np.ones((c, c), dtype=bool))
    A = np.where(lower, np.exp(np.where(lower, diff, 0.0)), 0.0)
    A_strict = np.tril(A, -1)
    L = beta[:, None] * (A_strict * (k @ k.T))
    return beta, g, A, L


def kla_chunkwise_unit(q, k, v, log_alpha, eta, eps, h0=None, chunk=64, want=False):
    """One (sequence, head): q,k [T,dk], v [T,dv], gates [T], h0 [dk,dv] or None.

    Returns (o [T,dv], hT [dk,dv]) and, if want, a list with one dict per chunk
    holding beta, g, L, T=(I+L)^-1, P=A o QK^T, U, W, U0, S_in.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    T_len, dk = k.shape
    dv = v.shape[1]
    S = np.zeros((dk, dv)) if h0 is None else np.array(h0, dtype=np.float64)
    o = np.zeros((T_len, dv))
    inter = []
    for c0 in range(0, T_len, chunk):
        c1 = min(T_len, c0 + chunk)
        K, V, Q = k[c0:c1], v[c0:c1], q[c0:c1]
        beta, g, A, L = chunk_objects(K, log_alpha[c0:c1], eta[c0:c1], eps)
        c = c1 - c0
        gam = np.exp(g)
        M = np.eye(c) + L
        rhs = beta[:, None] * (V - gam[:, None] * (K @ S))            # eq. (6) right-hand side
        U = solve_triangular(M, rhs, lower=True, unit_diagonal=True)  # eq. (6)
        P = A * (Q @ K.T)
        o[c0:c1] = gam[:, None] * (Q @ S) + P @ U                     # eq. (7)
        if want:
            Tm = solve_triangular(M, np.eye(c), lower=True, unit_diagonal=True)
            inter.append(dict(beta=beta, g=g, L=L, T=Tm, P=P, U=U, S_in=S.copy(),
                              W=Tm @ ((beta * gam)[:, None] * K), U0=Tm @ (beta[:, None] * V)))
        tail = np.exp(g[-1] - g)                                      # gamma_C / gamma_i
        S = gam[-1] * S + K.T @ (tail[:, None] * U)                   # eq. (8)
    if want:
        return o, S, inter
    return o, S


def kla_chunkwise(q, k, v, log_alpha, eta, eps, h0=None, cu_seqlens=None, chunk=64):
    """Batch front end with the same conventions as token_oracle.kla_recurrent."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    la = np.asarray(log_alpha, dtype=np.float64)
    et = np.asarray(eta, dtype=np.float64)
    N, T, H, dk = q.shape
    dv = v.shape[-1]
    if cu_seqlens is None:
        spans = [(n, 0, T) for n in range(N)]
    else:
        assert N == 1
        cu = [int(x) for x in cu_seqlens]
        spans = [(0, cu[i], cu[i + 1]) for i in range(len(cu) - 1)]
    o = np.zeros((N, T, H, dv))
    hT = np.zeros((len(spans), H, dk, dv))
    for s, (n, a, b) in enumerate(spans):
        for h in range(H):
            oo, ss = kla_chunkwise_unit(q[n, a:b, h], k[n, a:b, h], v[n, a:b, h], la[n, a:b, h],
                                        et[n, a:b, h], eps, None if h0 is None else h0[s, h], chunk)
            o[n, a:b, h] = oo
            hT[s, h] = ss
    return o, hT


def kla_chunkwise_bwd_unit(q, k, v, log_alpha, eta, eps, d_o, h0=None, d_hT=None, chunk=64, want=False):
    """Gradient of L = <d_o, o> + <d_hT, hT> for one (sequence, head), chunk by chunk.

    The paper gives no backward pass; this is eqs. (6)-(8) differentiated by hand, written per chunk with
    M = (I + L)^-1, X = V - D_gamma K S_in, U = M B X and the outgoing-state gradient dS':
        dU   = P^T dO + diag(gamma_C/gamma_i) K dS'          Y = M^T dU        dX = B Y   (= dV)
        dS_in = gamma_C dS' + Q^T D_gamma dO - K^T D_gamma dX
        dP   = tril(dO U^T)        dL = -tril(Y U^T, -1)        dbeta_i = Y_i.X_i + sum_j dL_ij A_ij (K K^T)_ij
        dQ   = D_gamma dO S_in^T + (A o dP) K
        dK   = -D_gamma dX S_in^T + diag(gamma_C/gamma_i) U dS'^T + (A o dP)^T Q + (D + D^T) K - 2 beta dbeta/(|k|^2+eps) k
               with D_ij = beta_i A_ij dL_ij
        dg_i = [every place g_i enters: D_gamma in X and O, A in P and L, gamma_C and gamma_C/gamma_i in eq. (8)]
        dlog_alpha_r = sum_{i >= r in the chunk} dg_i,     deta_i = dbeta_i / (|k_i|^2 + eps)
    It is pinned against the token-by-token gradient oracle in tests/test_oracle_pins.py.
    Returns a dict (dq, dk, dv, dlog_alpha, deta, dh0) and, if want, the per-chunk intermediates.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    la = np.asarray(log_alpha, dtype=np.float64)
    et = np.asarray(eta, dtype=np.float64)
    go = np.asarray(d_o, dtype=np.float64)
    T_len, dk = k.shape
    dv = v.shape[1]
    _, _, inter = kla_chunkwise_unit(q, k, v, la, et, eps, h0, chunk, want=True)
    dS = np.zeros((dk, dv)) if d_hT is None else np.array(d_hT, dtype=np.float64)
    out = dict(dq=np.zeros((T_len, dk)), dk=np.zeros((T_len, dk)), dv=np.zeros((T_len, dv)),
               dlog_alpha=np.zeros(T_len), deta=np.zeros(T_len))
    keep = []
    starts = list(range(0, T_len, chunk))
    for ci in reversed(range(len(starts))):
        c0 = starts[ci]
        c1 = min(T_len, c0 + chunk)
        K, V, Q, dO = k[c0:c1], v[c0:c1], q[c0:c1], go[c0:c1]
        it = inter[ci]
        beta, g, M, P, U, S_in = it["beta"], it["g"], it["T"], it["P"], it["U"], it["S_in"]
        c = c1 - c0
        gam = np.exp(g)
        tail = np.exp(g[-1] - g)
        lower = np.tril(np.ones((c, c), dtype=bool))
        A = np.where(lower, np.exp(np.where(lower, g[:, None] - g[None, :], 0.0)), 0.0)
        G = K @ K.T
        X = V - gam[:, None] * (K @ S_in)
        dU = P.T @ dO + tail[:, None] * (K @ dS)
        Y = M.T @ dU
        dX = beta[:, None] * Y
        dP = np.tril(dO @ U.T)
        dL = -np.tril(Y @ U.T, -1)
        dbeta = np.sum(Y * X, axis=1) + np.sum(dL * A * G, axis=1)
        D = beta[:, None] * A * dL
        den = np.sum(K * K, axis=1) + eps
        inv_den = np.where(den == 0.0, 0.0, 1.0 / np.where(den == 0.0, 1.0, den))
        dQ = gam[:, None] * (dO @ S_in.T) + (A * dP) @ K
        dK_read = -gam[:, None] * (dX @ S_in.T) + D @ K                    # k_i acting with gamma_i (rows of L, of X)
        dK_write = tail[:, None] * (U @ dS.T) + (A * dP).T @ Q + D.T @ K   # k_j acting with 1/gamma_j
        dK = dK_read + dK_write - (2.0 * beta * dbeta * inv_den)[:, None] * K
        # g_i multiplies q_i and the reading k_i, and divides the writing k_i; g_C enters eq. (8) twice more
        dg = np.sum(dQ * Q, axis=1) + np.sum(dK_read * K, axis=1) - np.sum(dK_write * K, axis=1)
        dg[-1] += gam[-1] * np.sum(dS * S_in) + np.sum((tail[:, None] * (U @ dS.T)) * K)
        out["dq"][c0:c1] = dQ
        out["dk"][c0:c1] = dK
        out["dv"][c0:c1] = dX
        out["deta"][c0:c1] = dbeta * inv_den
        out["dlog_alpha"][c0:c1] = np.cumsum(dg[::-1])[::-1]
        if want:
            keep.append(dict(dS_out=dS.copy(), dU=dU, Y=Y, X=X, dP=dP, dL=dL, dbeta=dbeta, dg=dg))
        dS = gam[-1] * dS + Q.T @ (gam[:, None] * dO) - K.T @ (gam[:, None] * dX)
    out["dh0"] = dS
    if want:
        return out, keep[::-1]
    return out


def kla_chunkwise_diag_unit(q, k, v, log_alpha, eta, eps, h0=None, chunk=64, want=False):
    """Chunkwise form with diagonal gating (App. B, "Extension to diagonal gating") for one (sequence, head).

    log_alpha is [T, dk].  gamma_i becomes a vector (running product of alpha per key channel, restarting at each
    chunk) and every decay ratio acts elementwise inside the inner products:
        L_ij = beta_i sum_c k_ic k_jc gamma_ic/gamma_jc  (j < i),     P_ij = sum_c q_ic k_jc gamma_ic/gamma_jc  (j <= i)
        (I + L) U = B (V - (K o Gamma) S_0),     O = (Q o Gamma) S_0 + P U,
        S_out = diag(gamma_C) S_0 + (K o (gamma_C / Gamma))^T U.
    The ratios are formed as exp of differences of the running log sums.  Returns (o, hT) and, if want, the per-chunk
    T = (I + L)^-1, P, beta and g.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    la = np.asarray(log_alpha, dtype=np.float64)
    et = np.asarray(eta, dtype=np.float64)
    T_len, dk = k.shape
    dv = v.shape[1]
    S = np.zeros((dk, dv)) if h0 is None else np.array(h0, dtype=np.float64)
    o = np.zeros((T_len, dv))
    inter = []
    for c0 in range(0, T_len, chunk):
        c1 = min(T_len, c0 + chunk)
        K, V, Q = k[c0:c1], v[c0:c1], q[c0:c1]
        c = c1 - c0
        g = np.cumsum(la[c0:c1], axis=0)                                   # [c, dk]
        den = np.sum(K * K, axis=1) + eps
        beta = np.where(den == 0.0, 0.0, et[c0:c1] / np.where(den == 0.0, 1.0, den))
        ratio = np.exp(np.minimum(g[:, None, :] - g[None, :, :], 0.0))     # [i, j, channel]; only j <= i is used
        KK = np.einsum("ic,jc,ijc->ij", K, K, ratio)
        QK = np.einsum("ic,jc,ijc->ij", Q, K, ratio)
        L = beta[:, None] * np.tril(KK, -1)
        P = np.tril(QK)
        gam = np.exp(g)
        rhs = beta[:, None] * (V - (K * gam) @ S)
        U = solve_triangular(np.eye(c) + L, rhs, lower=True, unit_diagonal=True)
        o[c0:c1] = (Q * gam) @ S + P @ U
        if want:
            inter.append(dict(beta=beta, g=g, P=P, T=solve_triangular(np.eye(c) + L, np.eye(c), lower=True, unit_diagonal=True)))
        S = gam[-1][:, None] * S + (K * np.exp(g[-1][None, :] - g)).T @ U
    if want:
        return o, S, inter
    return o, S
