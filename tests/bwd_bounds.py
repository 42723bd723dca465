"""Derived error bounds for the two gradients that the chunkwise backward forms as sums whose terms cancel.

Every other gradient is a sum of same-sized terms and meets the plain bars (1e-4 fp32, 2e-2 bf16).  Two are not:

* d eta_i = d beta_i / (|k_i|^2 + eps), d beta_i = Y_i . X_i + sum_j dL_ij A_ij (k_i . k_j).  With bf16 inputs the
  kernels keep Y, X, U and D' = -A^- o (Y U^T) in bf16 between their stages (unit roundoff u = 2^-9 each), so to first
  order |delta d beta_i| <= 2 u sum_c |Y_ic X_ic| + 3 u sum_j |dL_ij A_ij G_ij|.  On a tensor of a handful of entries,
  all of them sums over d_v products that mostly cancel, that can exceed 2e-2 of the largest entry.
* d log alpha_r = sum_{i >= r} dg_i, dg_i = q_i . dQ_i + k_i . dK^read_i - k_i . dK^write_i (see the chunkwise gradient
  oracle): where the decay wipes the state out within a token or two, the three inner products stay O(1) while their
  sum becomes far smaller, and fp32 rounding of the parts (unit roundoff 2^-24, a few hundred products per entry) is
  then large relative to the result although it is small relative to what was summed.  The scale of the parts,
  s_r = sum_{i >= r in the chunk} (|q_i . dQ_i| + |k_i . dK^read_i| + |k_i . dK^write_i|), is the yardstick: the fp32
  path is held to 1e-4 of max(max|d log alpha|, max s_r).

The functions below evaluate the bound and the scale in fp64 from the chunkwise oracle's intermediates.
"""
import numpy as np

from oracle import chunk_oracle


def _unit_bounds(q, k, v, la, eta, eps, d_o, h0, d_hT, u_in):
    q, k, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, k, v, d_o))
    T_len, dk = k.shape
    dv = v.shape[1]
    _, _, inter = chunk_oracle.kla_chunkwise_unit(q, k, v, la, eta, eps, h0, 64, want=True)
    _, keep = chunk_oracle.kla_chunkwise_bwd_unit(q, k, v, la, eta, eps, d_o, h0, d_hT, 64, want=True)
    b_eta = np.zeros(T_len)
    b_la = np.zeros(T_len)
    for ci, c0 in enumerate(range(0, T_len, 64)):
        c1 = min(T_len, c0 + 64)
        K, Q, dO = np.abs(k[c0:c1]), np.abs(q[c0:c1]), np.abs(d_o[c0:c1])
        it, kp = inter[ci], keep[ci]
        beta, g, U, S_in = it["beta"], it["g"], np.abs(it["U"]), np.abs(it["S_in"])
        Y, X, dS = np.abs(kp["Y"]), np.abs(kp["X"]), np.abs(kp["dS_out"])
        c = c1 - c0
        gam, tail = np.exp(g), np.exp(g[-1] - g)
        lower = np.tril(np.ones((c, c), dtype=bool))
        A = np.where(lower, np.exp(np.where(lower, g[:, None] - g[None, :], 0.0)), 0.0)
        G = np.abs(k[c0:c1] @ k[c0:c1].T)
        den = np.sum(K * K, axis=1) + eps
        inv_den = np.where(den == 0.0, 0.0, 1.0 / np.where(den == 0.0, 1.0, den))
        b_eta[c0:c1] = inv_den * (2 * u_in * np.sum(Y * X, axis=1) + 3 * u_in * np.sum(np.abs(kp["dL"]) * A * G, axis=1))
        # the three inner products of dg_i, signed, as the chunkwise oracle forms them
        Ks, Qs, dOs, Us, Ss, dSs = k[c0:c1], q[c0:c1], d_o[c0:c1], it["U"], it["S_in"], kp["dS_out"]
        dX = beta[:, None] * kp["Y"]
        Dm = beta[:, None] * A * kp["dL"]
        dQ = gam[:, None] * (dOs @ Ss.T) + (A * kp["dP"]) @ Ks
        dKr = -gam[:, None] * (dX @ Ss.T) + Dm @ Ks
        dKw = tail[:, None] * (Us @ dSs.T) + (A * kp["dP"]).T @ Qs + Dm.T @ Ks
        parts = np.abs(np.sum(dQ * Qs, axis=1)) + np.abs(np.sum(dKr * Ks, axis=1)) + np.abs(np.sum(dKw * Ks, axis=1))
        parts[-1] += abs(gam[-1] * np.sum(dSs * Ss)) + abs(np.sum((tail[:, None] * (Us @ dSs.T)) * Ks))
        b_la[c0:c1] = np.cumsum(parts[::-1])[::-1]
    return b_eta, b_la


def bounds(d, d_o, d_hT, to_f64, u_in=2.0 ** -9):
    """(bound on |delta d eta| with bf16 intermediates, scale s of the parts of d log alpha) as arrays shaped like eta,
    for a batch dict of kla_inputs (fixed-length or packed); to_f64 widens a tensor exactly."""
    q, k, v, go = [to_f64(d[x]) for x in "qkv"] + [to_f64(d_o)]
    la, et = d["log_alpha"].double().numpy(), d["eta"].double().numpy()
    N, T, H = la.shape
    be, bl = np.zeros((N, T, H)), np.zeros((N, T, H))
    cu = None if d["cu_seqlens"] is None else d["cu_seqlens"].numpy()
    n_seq = N if cu is None else len(cu) - 1
    for s in range(n_seq):
        n, t0, t1 = (s, 0, T) if cu is None else (0, int(cu[s]), int(cu[s + 1]))
        if t1 == t0:
            continue
        for h in range(H):
            h0 = None if d["h0"] is None else d["h0"][s, h].double().numpy()
            g = None if d_hT is None else d_hT[s, h].double().numpy()
            e, l = _unit_bounds(q[n, t0:t1, h], k[n, t0:t1, h], v[n, t0:t1, h], la[n, t0:t1, h], et[n, t0:t1, h], d["eps"],
                                go[n, t0:t1, h], h0, g, u_in)
            be[n, t0:t1, h], bl[n, t0:t1, h] = e, l
    return be, bl
