"""Chunkwise fp64 model of the gated OSDN pass (numpy) -- test helper.

An independent second implementation used to pin the token-by-token oracle
("recurrent and chunkwise forms must agree") and to validate the chunk-level
backward algebra.  Forward follows the chunkwise WY derivation (Appendix A.2)
in the decay-ratio gauge of Appendix B.1:

    A_ij = 1[j<i] beta_i (gamma_i/gamma_j) <k_i, k~_j>,   T = (I + A)^-1,
    W = T diag(beta) (gamma . K),  U = T diag(beta) V,  E = U - W S^T,
    O = scale [ (gamma . Q) S^T + tril(Gamma . Q K~^T) E ],
    S' = gamma_C S + E^T (rho . K~),  rho_i = gamma_C / gamma_i.

Only pairwise ratios exp(G_i - G_j) with j <= i (all <= 1) are ever formed.
The backward is ordinary matrix calculus on those formulas (the paper prints
only the chain rule through k~ = d . k, Section 4.5).
"""
import numpy as np
from scipy.linalg import solve_triangular


def _chunk_quantities(Q, K, Kt, V, beta, g, S):
    C = K.shape[0]
    G = np.cumsum(g)
    diff = G[:, None] - G[None, :]
    low = np.tril(np.ones((C, C), dtype=bool))
    Gam = np.where(low, np.exp(np.where(low, diff, 0.0)), 0.0)      # j <= i
    gam = np.exp(G)
    rho = np.exp(G[-1] - G)
    KKt = K @ Kt.T
    A0 = np.tril(Gam * KKt, -1)
    A = beta[:, None] * A0
    Tm = solve_triangular(np.eye(C) + A, np.eye(C), lower=True, unit_diagonal=True)
    R0 = V - (gam[:, None] * K) @ S.T
    E = Tm @ (beta[:, None] * R0)
    QKt = Q @ Kt.T
    P = Gam * QKt                                                   # tril incl. diagonal
    return dict(G=G, Gam=Gam, gam=gam, rho=rho, KKt=KKt, A0=A0, A=A, Tm=Tm, R0=R0, E=E,
                QKt=QKt, P=P)


def chunk_fwd_chain(q, k, kt, v, beta, g, S0, scale, C=64, keep=False):
    """One (b,h) chain.  q,k,kt [T,K]; v [T,V]; beta,g [T]; S0 [V,K]."""
    T = q.shape[0]
    assert T % C == 0
    S = S0.copy()
    o = np.empty((T, v.shape[1]))
    states = []
    for n in range(T // C):
        sl = slice(n * C, (n + 1) * C)
        c = _chunk_quantities(q[sl], k[sl], kt[sl], v[sl], beta[sl], g[sl], S)
        if keep:
            states.append(S.copy())
        o[sl] = scale * ((c["gam"][:, None] * q[sl]) @ S.T + c["P"] @ c["E"])
        S = c["gam"][-1] * S + c["E"].T @ (c["rho"][:, None] * kt[sl])
    return (o, S, states) if keep else (o, S)


def chunk_bwd_chain(q, k, kt, v, beta, g, S0, scale, dO, dS_T, C=64):
    """Backward of chunk_fwd_chain w.r.t. q, k (read side), kt (write side), v,
    beta, g, S0.  Returns dq, dk, dkt, dv, dbeta, dg, dS0."""
    T = q.shape[0]
    N = T // C
    _, _, states = chunk_fwd_chain(q, k, kt, v, beta, g, S0, scale, C, keep=True)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dkt = np.zeros_like(kt)
    dv = np.zeros_like(v); dbeta = np.zeros_like(beta); dg = np.zeros_like(g)
    dS = dS_T.copy()                       # adjoint of the state at the END of the chunk
    for n in range(N - 1, -1, -1):
        sl = slice(n * C, (n + 1) * C)
        Q, K, Kt, V_, b, S = q[sl], k[sl], kt[sl], v[sl], beta[sl], states[n]
        c = _chunk_quantities(Q, K, Kt, V_, b, g[sl], S)
        gam, rho, Gam, Tm, E = c["gam"], c["rho"], c["Gam"], c["Tm"], c["E"]
        dOc = dO[sl]
        # --- the part carried along the chain ---
        dE = scale * c["P"].T @ dOc + (rho[:, None] * Kt) @ dS.T
        dR = Tm.T @ dE                                   # adjoint of R = beta . R0
        W = Tm @ (b[:, None] * gam[:, None] * K)
        dS_prev = gam[-1] * dS + scale * dOc.T @ (gam[:, None] * Q) - dE.T @ W
        # --- everything else ---
        dP = scale * np.tril(dOc @ E.T)
        dQg = scale * dOc @ S                            # adjoint of gamma . Q
        dKr = E @ dS                                     # adjoint of rho . K~
        dKg = -(b[:, None] * dR) @ S                     # adjoint of gamma . K
        dA = -np.tril(dR @ E.T, -1)
        dv[sl] = b[:, None] * dR
        dbeta[sl] = (dR * c["R0"]).sum(1) + (dA * c["A0"]).sum(1)
        cA = dA * b[:, None] * Gam
        cP = dP * Gam
        dk[sl] = cA @ Kt + gam[:, None] * dKg
        dkt[sl] = cA.T @ K + cP.T @ Q + rho[:, None] * dKr
        dq[sl] = cP @ Kt + gam[:, None] * dQg
        X = dA * c["A"] + dP * c["P"]
        rk = (dKr * rho[:, None] * Kt).sum(1)
        dG = X.sum(1) - X.sum(0) + (dQg * gam[:, None] * Q).sum(1) \
            + (dKg * gam[:, None] * K).sum(1) - rk
        dG[-1] += rk.sum() + gam[-1] * (dS * S).sum()
        dg[sl] = np.cumsum(dG[::-1])[::-1]
        dS = dS_prev
    return dq, dk, dkt, dv, dbeta, dg, dS
