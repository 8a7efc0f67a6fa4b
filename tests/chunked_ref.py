"""fp64 numpy model of the chunked (state-space-duality) algorithm the HIP kernels implement.

Test infrastructure: it exists to prove, on the CPU, that the chunked forward and backward
formulas the kernels are built from equal the token-by-token recurrence (the oracle), for any
chunk and segment size.  It is neither the oracle nor the product.

Per (batch, head), per chunk of Q tokens with entering state Hprev, local index i, j in [0, Q):
    a_j = dt_j A,  cum_i = sum_{r<=i} a_r,  T = cum_{Q-1},  G[i,j] = C_i.B_j
    S      = sum_j exp(T - cum_j) dt_j x_j (x) B_j            Hnext = exp(T) Hprev + S
    yhat_i = sum_{j<=i} G[i,j] exp(cum_i - cum_j) dt_j x_j + exp(cum_i) Hprev C_i      y = yhat + D x
backward, given dY and dHnext:
    dHprev = exp(T) dHnext + sum_i exp(cum_i) dY_i (x) C_i
    u_j    = sum_{i>=j} G[i,j] exp(cum_i - cum_j) dY_i + exp(T - cum_j) dHnext B_j     dx_j = dt_j u_j + D dY_j
    W[i,j] = exp(cum_i - cum_j) dt_j (dY_i . x_j)   (j <= i),   dG = sum over the group's heads of W
    dC_i   = sum_j dG[i,j] B_j + sum_heads exp(cum_i) dY_i^T Hprev
    dB_j   = sum_i dG[i,j] C_i + sum_heads exp(T - cum_j) dt_j x_j^T dHnext
    da_r   = sum_{i>=r} (dY_i . yhat_i - dt_i x_i . u_i) + <dHnext, Hnext>
    ddt_j  = A da_j + x_j . u_j,   dA += sum_j dt_j da_j,   dD += sum dY . x
"""
import numpy as np


def forward(x, dt, A, Bm, Cm, D, Q, init_state=None):
    Bt, L, H, P = x.shape
    G, N = Bm.shape[2:]
    nc = L // Q
    y = np.zeros_like(x)
    entering = np.zeros((Bt, nc + 1, H, P, N))
    cum_all = np.zeros((Bt, H, nc, Q))
    for b in range(Bt):
        for h in range(H):
            g = h // (H // G)
            Hs = np.zeros((P, N)) if init_state is None else init_state[b, h].copy()
            for c in range(nc):
                sl = slice(c * Q, (c + 1) * Q)
                X, d, Bc, Cc = x[b, sl, h], dt[b, sl, h], Bm[b, sl, g], Cm[b, sl, g]
                cum = np.cumsum(d * A[h])
                T = cum[-1]
                cum_all[b, h, c] = cum
                entering[b, c, h] = Hs
                M = np.tril((Cc @ Bc.T) * np.exp(np.minimum(cum[:, None] - cum[None, :], 0.0))) * d[None, :]
                y[b, sl, h] = M @ X + np.exp(cum)[:, None] * (Cc @ Hs.T) + D[h] * X
                S = np.einsum("j,jp,jn->pn", np.exp(T - cum) * d, X, Bc)
                Hs = np.exp(T) * Hs + S
            entering[b, nc, h] = Hs
    return y, entering, cum_all


def backward(x, dt, A, Bm, Cm, D, dy, Q, entering, dfinal=None):
    Bt, L, H, P = x.shape
    G, N = Bm.shape[2:]
    nc = L // Q
    dx, ddt = np.zeros_like(x), np.zeros_like(dt)
    dB, dC = np.zeros_like(Bm), np.zeros_like(Cm)
    dA, dD = np.zeros(H), np.zeros(H)
    dinit = np.zeros((Bt, H, P, N))
    for b in range(Bt):
        for h in range(H):
            g = h // (H // G)
            dHnext = np.zeros((P, N)) if dfinal is None else dfinal[b, h].copy()
            for c in range(nc - 1, -1, -1):
                sl = slice(c * Q, (c + 1) * Q)
                X, d, Bc, Cc, dY = x[b, sl, h], dt[b, sl, h], Bm[b, sl, g], Cm[b, sl, g], dy[b, sl, h]
                Hprev, Hnext = entering[b, c, h], entering[b, c + 1, h]
                cum = np.cumsum(d * A[h])
                T = cum[-1]
                dec = np.tril(np.exp(np.minimum(cum[:, None] - cum[None, :], 0.0)))
                Gm = Cc @ Bc.T
                w = np.exp(T - cum)
                yhat = (Gm * dec * d[None, :]) @ X + np.exp(cum)[:, None] * (Cc @ Hprev.T)
                u = (Gm * dec).T @ dY + w[:, None] * (Bc @ dHnext.T)
                dx[b, sl, h] = d[:, None] * u + D[h] * dY
                W = dec * d[None, :] * (dY @ X.T)
                dC[b, sl, g] += W @ Bc + np.exp(cum)[:, None] * (dY @ Hprev)
                dB[b, sl, g] += W.T @ Cc + (w * d)[:, None] * (X @ dHnext)
                term = np.sum(dY * yhat, 1) - d * np.sum(X * u, 1)
                da = np.cumsum(term[::-1])[::-1] + np.sum(dHnext * Hnext)
                ddt[b, sl, h] = A[h] * da + np.sum(X * u, 1)
                dA[h] += np.sum(d * da)
                dD[h] += np.sum(dY * X)
                dHnext = np.exp(T) * dHnext + np.einsum("i,ip,in->pn", np.exp(cum), dY, Cc)
            dinit[b, h] = dHnext
    return dict(dx=dx, ddt=ddt, dA=dA, dB=dB, dC=dC, dD=dD, dinit_state=dinit)
