"""Brute-force, partition-free statement of the compressed layer, used to pin the step-by-step oracle.

With part(i) the owner of node i, S_intra = S * [part(i) == part(j)], S_cross = S - S_intra and Mask the
n x F keep-mask of the layer's input (k ones per row), all partitions at once compute

    M     = S_intra X + S_cross (Mask * X)
    X_out = rho(M H1 + X H0)
    dZ    = dX_out * rho'(.) ; dH1 = M^T dZ ; dH0 = X^T dZ ; dM = dZ H1^T
    dX    = S_intra^T dM + Mask * (S_cross^T dM) + dZ H0^T

At ratio 1 (Mask = 1) this is eq. (2) of the paper on the unpartitioned graph: rho(S X H1 + X H0).
Dense numpy only; nothing here touches the oracle's partition structures.
"""
import numpy as np


def dense_operator(g):
    s = np.zeros((g.n, g.n), dtype=np.float64)
    for i in range(g.n):
        for e in range(g.rowptr[i], g.rowptr[i + 1]):
            s[i, g.colidx[e]] += float(g.vals[e])
    return s


def split_operator(s, part):
    same = part[:, None] == part[None, :]
    return s * same, s * (~same)


def forward(s_intra, s_cross, mask, x, h1, h0, relu):
    m = s_intra @ x + s_cross @ (mask * x)
    zpre = m @ h1 + (x @ h0 if h0 is not None else 0.0)
    return (np.maximum(zpre, 0.0) if relu else zpre), m


def backward(s_intra, s_cross, mask, x, m, x_out, dx_out, h1, h0, relu):
    dz = dx_out * (x_out > 0) if relu else dx_out
    dh1 = m.T @ dz
    dh0 = x.T @ dz if h0 is not None else None
    dm = dz @ h1.T
    dx = s_intra.T @ dm + mask * (s_cross.T @ dm)
    if h0 is not None:
        dx = dx + dz @ h0.T
    return dh1, dh0, dx
