"""Row-at-a-time evaluation of the compressed layer for chosen nodes (oracle side; test infrastructure).

For graphs too large to run the whole step-by-step oracle in seconds, single output rows can still be
computed exactly from their definition on the global graph (eq. (2) with the partition and the keep-mask
applied to remote neighbours, Algorithm 1):

    M[v]      = sum_c S[v,c] * ( X[c]            if part(c) == part(v)
                                 mask_c * X[c]    otherwise )
    X_out[v]  = rho( M[v] H1 + X[v] H0 )
    dX[v]     = sum_{i: part(i)==part(v)} S[i,v] dM[i]  +  mask_v * sum_{i: part(i)!=part(v)} S[i,v] dM[i]
                + dZ[v] H0^T,          dM[i] = dZ[i] H1^T,  dZ[i] = dX_out[i] * [X_out[i] > 0]
    returned to v's owner by consumer q:  ( sum_{i in q} S[i,v] dM[i] ) at v's kept positions

Everything in fp64, entry by entry; pinned against the step-by-step oracle on small graphs.
"""
from __future__ import annotations

import numpy as np

from . import mask as _mask


def forward_rows(rowptr, colidx, vals, part, x, nodes, k, key, step, layer, h1, h0, relu):
    """(M[nodes], X_out[nodes]) from the global CSR of S, the node->partition map and the layer input x."""
    width = x.shape[1]
    h1 = np.asarray(h1, dtype=np.float64)
    m_out = np.empty((len(nodes), width))
    for n, v in enumerate(nodes):
        cols = np.asarray(colidx[rowptr[v]:rowptr[v + 1]], dtype=np.int64)
        w = np.asarray(vals[rowptr[v]:rowptr[v + 1]], dtype=np.float64)
        xr = np.asarray(x[cols], dtype=np.float64)
        remote = part[cols] != part[v]
        if remote.any():
            xr[remote] *= _mask.keep_mask(cols[remote], width, k, key, step, layer)
        m_out[n] = w @ xr
    zpre = m_out @ h1
    if h0 is not None:
        zpre = zpre + np.asarray(x[np.asarray(nodes)], dtype=np.float64) @ np.asarray(h0, dtype=np.float64)
    return m_out, (np.maximum(zpre, 0.0) if relu else zpre)


def _dm_rows(rows, dx_out, x_out, h1, relu):
    dz = np.asarray(dx_out[rows], dtype=np.float64)
    if relu:
        dz = dz * (np.asarray(x_out[rows]) > 0)
    return dz @ np.asarray(h1, dtype=np.float64).T


def backward_rows(t_rowptr, t_colidx, t_vals, part, dx_out, x_out, nodes, k, key, step, layer, h1, h0, relu):
    """dX[nodes]. (t_rowptr, t_colidx, t_vals) is the CSR of S^T: row v lists (i, S[i, v])."""
    width = h1.shape[0]
    out = np.empty((len(nodes), width))
    for n, v in enumerate(nodes):
        rows = np.asarray(t_colidx[t_rowptr[v]:t_rowptr[v + 1]], dtype=np.int64)
        w = np.asarray(t_vals[t_rowptr[v]:t_rowptr[v + 1]], dtype=np.float64)
        dm = _dm_rows(rows, dx_out, x_out, h1, relu)
        same = part[rows] == part[v]
        acc = w[same] @ dm[same]
        if (~same).any():
            acc = acc + _mask.keep_mask(np.array([v]), width, k, key, step, layer)[0] * (w[~same] @ dm[~same])
        if h0 is not None:
            dz = np.asarray(dx_out[v], dtype=np.float64)
            if relu:
                dz = dz * (np.asarray(x_out[v]) > 0)
            acc = acc + dz @ np.asarray(h0, dtype=np.float64).T
        out[n] = acc
    return out


def returned_rows(t_rowptr, t_colidx, t_vals, part, dx_out, x_out, consumer, nodes, k, key, step, layer, h1, relu):
    """What consumer partition `consumer` hands back for the (remote) nodes: [len(nodes), k]."""
    width = h1.shape[0]
    cols = _mask.kept_columns(np.asarray(nodes), width, k, key, step, layer)
    out = np.empty((len(nodes), k))
    for n, v in enumerate(nodes):
        rows = np.asarray(t_colidx[t_rowptr[v]:t_rowptr[v + 1]], dtype=np.int64)
        w = np.asarray(t_vals[t_rowptr[v]:t_rowptr[v + 1]], dtype=np.float64)
        sel = part[rows] == consumer
        dm = _dm_rows(rows[sel], dx_out, x_out, h1, relu)
        out[n] = (w[sel] @ dm)[cols[n]]
    return out
