"""One partition's layer step, forward and backward (oracle side; test infrastructure).

Follows Algorithm 1 for a single layer l of eq. (2), X_l = rho( sum_k S^k X_{l-1} H_{l,k} ), with the
taps the experiments use (Section V): a single tap S (GCN-style) or the taps I and S (SAGE):

  forward   owners compress the boundary rows of X_{l-1} (Definition 1, Appendix "Compression
            Mechanism"): Z = the k kept elements of each row
            consumer q decompresses its halo rows: kept elements in place, zero elsewhere, no rescale
            M     = S_q [X_loc ; X~_halo]                       (uncompressed local, compressed remote)
            Zpre  = M H_1 (+ X_loc H_0)
            X_out = rho(Zpre),  rho = ReLU or identity
  backward  (the exact gradient of the forward above with the kept positions frozen)
            dZ = dX_out * [X_out > 0]           (identity layer: dZ = dX_out)
            dH_1 = M^T dZ ;  dH_0 = X_loc^T dZ ;  dM = dZ H_1^T
            [dX_loc ; dX~_halo] = S_q^T dM ;  dX_loc += dZ H_0^T
            errors returned to owners: the same k positions of each halo row of dX~_halo
            owner:  dX[boundary row, kept positions] += returned values, summed over consumers

Everything is computed in fp64 on the inputs as given (fp32 or bf16 values are exactly representable).
"""
from __future__ import annotations

import numpy as np
import scipy.sparse as sp

from . import mask as _mask
from .partition import Partition

RELU = 1
IDENTITY = 0


def compress(x: np.ndarray, rows: np.ndarray, cols: np.ndarray) -> np.ndarray:
    """Z[i, j] = x[rows[i], cols[i, j]]."""
    rows = np.asarray(rows, dtype=np.int64)
    return np.asarray(x, dtype=np.float64)[rows[:, None], cols]


def decompress(z: np.ndarray, cols: np.ndarray, width: int) -> np.ndarray:
    """Rows of `width` elements: z's values at their kept positions, zero elsewhere."""
    out = np.zeros((z.shape[0], width), dtype=np.float64)
    out[np.arange(z.shape[0])[:, None], cols] = z
    return out


def scatter_add(x: np.ndarray, rows: np.ndarray, cols: np.ndarray, z: np.ndarray) -> None:
    """x[rows[i], cols[i, j]] += z[i, j]  (rows distinct; positions distinct within a row)."""
    rows = np.asarray(rows, dtype=np.int64)
    x[rows[:, None], cols] += z


def _block(p: Partition) -> sp.csr_matrix:
    return sp.csr_matrix((p.vals.astype(np.float64), p.colidx.astype(np.int64), p.rowptr.astype(np.int64)),
                         shape=(p.n_local, p.n_local + p.n_halo))


def layer_forward(p: Partition, x_local: np.ndarray, z_all: np.ndarray, halo_cols: np.ndarray,
                  h1: np.ndarray, h0, act: int, with_pre: bool = False):
    """Forward of one layer on partition `p`.

    x_local [n_local, F_in]; z_all: concatenated compressed boundary rows of all owners [sum b_p, k];
    halo_cols [n_halo, k]: kept positions of each halo node. Returns (x_out, m), both fp64; with_pre adds the
    argument of the nonlinearity, Zpre, as a third result.
    """
    x_local = np.asarray(x_local, dtype=np.float64)
    width = x_local.shape[1]
    z_halo = np.asarray(z_all, dtype=np.float64)[p.halo_zrow.astype(np.int64)]        # hand-off
    x_halo = decompress(z_halo, halo_cols, width)
    m = _block(p) @ np.vstack([x_local, x_halo])
    zpre = m @ np.asarray(h1, dtype=np.float64)
    if h0 is not None:
        zpre = zpre + x_local @ np.asarray(h0, dtype=np.float64)
    x_out = np.maximum(zpre, 0.0) if act == RELU else zpre
    return (x_out, m, zpre) if with_pre else (x_out, m)


def layer_backward(p: Partition, dx_out: np.ndarray, x_out: np.ndarray, x_local: np.ndarray, m: np.ndarray,
                   halo_cols: np.ndarray, h1: np.ndarray, h0, act: int, need_input_grad: bool = True):
    """Backward of one layer on partition `p`.

    Returns (dh1, dh0 or None, dx_local or None, dz_halo or None); dz_halo [n_halo, k] holds the halo
    rows' gradient at the kept positions only.
    """
    dx_out = np.asarray(dx_out, dtype=np.float64)
    dz = dx_out * (np.asarray(x_out) > 0) if act == RELU else dx_out
    m = np.asarray(m, dtype=np.float64)
    x_local = np.asarray(x_local, dtype=np.float64)
    dh1 = m.T @ dz
    dh0 = x_local.T @ dz if h0 is not None else None
    if not need_input_grad:
        return dh1, dh0, None, None
    dm = dz @ np.asarray(h1, dtype=np.float64).T
    dcat = _block(p).T @ dm
    dx_local = np.asarray(dcat[:p.n_local])
    if h0 is not None:
        dx_local = dx_local + dz @ np.asarray(h0, dtype=np.float64).T
    dx_halo = np.asarray(dcat[p.n_local:])
    dz_halo = dx_halo[np.arange(p.n_halo)[:, None], halo_cols]
    return dh1, dh0, dx_local, dz_halo


# ---------------------------------------------------------------------------------------------------
# all partitions in turn, all layers: one training step's forward and backward (Algorithm 1, without
# the loss and the parameter update)
# ---------------------------------------------------------------------------------------------------

# (network_step = network_forward + network_backward)

def network_forward(parts: list[Partition], x0: list[np.ndarray], weights: list[tuple], acts: list[int],
                    keep: list[int], key: int, step: int, round_store=None):
    """Forward over all layers and partitions. Returns the state network_backward needs: per-layer
    activations `x`, saved aggregates `m`, compressed buffers `z`, the arguments of the nonlinearity `zpre`
    (fp64, not rounded: what decides the ReLU gate) and the forward hand-off counts."""
    rnd = (lambda a: a) if round_store is None else round_store
    n_layers = len(weights)
    xs = [[np.asarray(x, dtype=np.float64) for x in x0]]
    ms, zs, pres = [], [], []
    fwd_elems = []
    for l in range(n_layers):
        width = xs[l][0].shape[1]
        k = keep[l]
        z_all = np.vstack([
            compress(xs[l][p.q], p.boundary_rows,
                     _mask.kept_columns(p.local_gid[p.boundary_rows], width, k, key, step, l))
            for p in parts])
        z_all = rnd(z_all)
        zs.append(z_all)
        out, agg, pre = [], [], []
        for p in parts:
            cols = _mask.kept_columns(p.halo_gid, width, k, key, step, l)
            xo, m, zpre = layer_forward(p, xs[l][p.q], z_all, cols, weights[l][0], weights[l][1], acts[l], True)
            out.append(rnd(xo))
            agg.append(rnd(m))
            pre.append(zpre)
        xs.append(out)
        ms.append(agg)
        pres.append(pre)
        fwd_elems.append(sum(p.n_halo for p in parts) * k)
    return dict(x=xs, m=ms, z=zs, zpre=pres, fwd_elems=fwd_elems)


def network_backward(parts: list[Partition], fwd: dict, weights: list[tuple], acts: list[int], keep: list[int],
                     key: int, step: int, dx_last: list[np.ndarray], round_store=None):
    """Backward over all layers and partitions from the upstream gradient of the last layer's output.
    Returns weight gradients (summed over partitions), input gradients per layer and hand-off counts."""
    rnd = (lambda a: a) if round_store is None else round_store
    xs, ms = fwd["x"], fwd["m"]
    n_layers = len(weights)
    n_parts = len(parts)
    bwd_elems = []
    dh = [[None, None] for _ in range(n_layers)]
    dx = list(dx_last)
    dxs = {n_layers: dx}
    for l in range(n_layers - 1, -1, -1):
        width = xs[l][0].shape[1]
        k = keep[l]
        need = l > 0
        new_dx = [None] * n_parts
        returned = []
        for p in parts:
            cols = _mask.kept_columns(p.halo_gid, width, k, key, step, l)
            dh1, dh0, dxl, dzh = layer_backward(p, dx[p.q], xs[l + 1][p.q], xs[l][p.q], ms[l][p.q], cols,
                                                weights[l][0], weights[l][1], acts[l], need)
            dh[l][0] = dh1 if dh[l][0] is None else dh[l][0] + dh1
            if dh0 is not None:
                dh[l][1] = dh0 if dh[l][1] is None else dh[l][1] + dh0
            if need:
                new_dx[p.q] = rnd(dxl)
                returned.append((p, cols, rnd(dzh)))
        if not need:
            bwd_elems.append(0)
            break
        # owners accumulate what came back, consumers in ascending order
        for (p, cols, dzh) in returned:
            for o in range(n_parts):
                s0, s1 = int(p.halo_owner_ptr[o]), int(p.halo_owner_ptr[o + 1])
                if s1 == s0:
                    continue
                rows = parts[o].boundary_rows[p.halo_src_row[s0:s1]]
                scatter_add(new_dx[o], rows, cols[s0:s1], dzh[s0:s1])
        new_dx = [rnd(a) for a in new_dx]
        dx = new_dx
        dxs[l] = dx
        bwd_elems.append(sum(p.n_halo for p in parts) * k)
    return dict(dh=dh, dx=dxs, bwd_elems=bwd_elems[::-1])


def network_step(parts: list[Partition], x0: list[np.ndarray], weights: list[tuple], acts: list[int],
                 keep: list[int], key: int, step: int, dx_last: list[np.ndarray],
                 round_store=None):
    """Forward then backward over all partitions.

    x0[q]: partition q's input rows. weights[l] = (H1, H0 or None). keep[l] = k of layer l's input.
    dx_last[q]: upstream gradient of the last layer's output. `round_store`, when given, is applied to
    every tensor at the point where the device path stores it (e.g. rounding to fp32 or bf16).

    Returns a dict with per-layer activations, saved aggregates, weight gradients, input gradients and the
    number of compressed elements handed off forward and backward per layer.
    """
    fwd = network_forward(parts, x0, weights, acts, keep, key, step, round_store)
    bwd = network_backward(parts, fwd, weights, acts, keep, key, step, dx_last, round_store)
    return dict(x=fwd["x"], m=fwd["m"], z=fwd["z"], zpre=fwd["zpre"], dh=bwd["dh"], dx=bwd["dx"], fwd_elems=fwd["fwd_elems"],
                bwd_elems=bwd["bwd_elems"])
