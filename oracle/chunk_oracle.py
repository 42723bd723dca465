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
