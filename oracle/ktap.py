"""General K-tap graph-convolution layer with a compressed exchange per hop (oracle side; test
infrastructure).

Eq. (1)-(2): X_l = rho( sum_{k=0}^{K-1} S^k X_{l-1} H_{l,k} ). With the graph partitioned (Section III), every
application of S needs the rows of adjacent partitions, so each hop k = 1..K-1 has an exchange of its own:

    Y_0 = X_{l-1};   owners compress the boundary rows of Y_{k-1} (positions of hop k), consumers decompress,
    Y_k = S_q [Y_{k-1,loc} ; Y~_{k-1,halo}],   k = 1..K-1;     X_l = rho( sum_k Y_k H_k )

and the backward pass runs the hops in reverse, handing the errors of halo rows back at every hop:

    dZ = dX_l * rho'(.);   dH_k = Y_k^T dZ;   G_{K-1} = dZ H_{K-1}^T
    for k = K-1 .. 1:   [C_loc ; C_halo] = S_q^T G_k;   the kept positions of C_halo go back to the owners;
                        G_{k-1} = dZ H_{k-1}^T + C_loc + (what the consumers returned, at its positions)
    dX_{l-1} = G_0

K = 2 is the two-tap (SAGE) layer of oracle/layer.py. The kept positions of hop k of layer l are those of
"layer index" l + 16 k of oracle/mask.py (hop 0 is never exchanged), so that every hop draws its own positions.
Everything in fp64.
"""
from __future__ import annotations

import numpy as np

from . import layer as _layer
from . import mask as _mask

HOP_STRIDE = 16


def tap(layer: int, hop: int) -> int:
    return layer + HOP_STRIDE * hop


def _exchange(parts, y, width, k, key, step, addr):
    """Owners compress, consumers pick their halo rows: returns (z_all, per-partition halo columns)."""
    z_all = np.vstack([_layer.compress(y[p.q], p.boundary_rows,
                                       _mask.kept_columns(p.local_gid[p.boundary_rows], width, k, key, step, addr))
                       for p in parts])
    cols = [_mask.kept_columns(p.halo_gid, width, k, key, step, addr) for p in parts]
    return z_all, cols


def layer_forward(parts, x, weights, act, k, key, step, layer):
    """x[q]: partition q's rows of X_{l-1}; weights = [H_0 .. H_{K-1}]. Returns (x_out per partition, ys) with
    ys[hop][q] = Y_hop rows of partition q (ys[0] = x)."""
    n_taps = len(weights)
    width = x[0].shape[1]
    ys = [[np.asarray(a, dtype=np.float64) for a in x]]
    for hop in range(1, n_taps):
        z_all, cols = _exchange(parts, ys[hop - 1], width, k, key, step, tap(layer, hop))
        nxt = []
        for p in parts:
            halo = _layer.decompress(z_all[p.halo_zrow.astype(np.int64)], cols[p.q], width)
            nxt.append(_layer._block(p) @ np.vstack([ys[hop - 1][p.q], halo]))
        ys.append(nxt)
    out = []
    for p in parts:
        zpre = sum(ys[hop][p.q] @ np.asarray(weights[hop], dtype=np.float64) for hop in range(n_taps))
        out.append(np.maximum(zpre, 0.0) if act == _layer.RELU else zpre)
    return out, ys


def layer_backward(parts, dx_out, x_out, ys, weights, act, k, key, step, layer, need_input_grad=True):
    """Returns (dh = [dH_0 .. dH_{K-1}] summed over partitions, dx per partition or None, elements handed back)."""
    n_taps = len(weights)
    n_parts = len(parts)
    width = ys[0][0].shape[1]
    dz = [np.asarray(dx_out[p.q], dtype=np.float64) * (np.asarray(x_out[p.q]) > 0) if act == _layer.RELU
          else np.asarray(dx_out[p.q], dtype=np.float64) for p in parts]
    dh = [sum(ys[hop][p.q].T @ dz[p.q] for p in parts) for hop in range(n_taps)]
    if not need_input_grad:
        return dh, None, 0
    g = [dz[p.q] @ np.asarray(weights[n_taps - 1], dtype=np.float64).T for p in parts]
    handed_back = 0
    for hop in range(n_taps - 1, 0, -1):
        addr = tap(layer, hop)
        nxt = [dz[p.q] @ np.asarray(weights[hop - 1], dtype=np.float64).T for p in parts]
        returned = []
        for p in parts:
            cat = _layer._block(p).T @ g[p.q]
            nxt[p.q] = nxt[p.q] + np.asarray(cat[:p.n_local])
            cols = _mask.kept_columns(p.halo_gid, width, k, key, step, addr)
            returned.append((p, cols, np.asarray(cat[p.n_local:])[np.arange(p.n_halo)[:, None], cols]))
        for (p, cols, dzh) in returned:          # owners add what came back, consumers in ascending order
            for o in range(n_parts):
                s0, s1 = int(p.halo_owner_ptr[o]), int(p.halo_owner_ptr[o + 1])
                if s1 > s0:
                    _layer.scatter_add(nxt[o], parts[o].boundary_rows[p.halo_src_row[s0:s1]], cols[s0:s1], dzh[s0:s1])
        handed_back += sum(p.n_halo for p in parts) * k
        g = nxt
    return dh, g, handed_back


def network_step(parts, x0, weights, acts, keep, key, step, dx_last):
    """All layers, forward then backward. weights[l] = [H_0 .. H_{K-1}]. Returns activations, hop aggregates,
    weight gradients, input gradients and the hand-off counts per layer (all hops of a layer added up)."""
    n_layers = len(weights)
    xs, yss, fwd_elems = [[np.asarray(a, dtype=np.float64) for a in x0]], [], []
    for l in range(n_layers):
        out, ys = layer_forward(parts, xs[l], weights[l], acts[l], keep[l], key, step, l)
        xs.append(out)
        yss.append(ys)
        fwd_elems.append(sum(p.n_halo for p in parts) * keep[l] * (len(weights[l]) - 1))
    dhs, dxs, bwd_elems = [None] * n_layers, {n_layers: list(dx_last)}, [0] * n_layers
    dx = list(dx_last)
    for l in range(n_layers - 1, -1, -1):
        dhs[l], dx, bwd_elems[l] = layer_backward(parts, dx, xs[l + 1], yss[l], weights[l], acts[l], keep[l], key, step,
                                                  l, need_input_grad=l > 0)
        if l > 0:
            dxs[l] = dx
    return dict(x=xs, y=yss, dh=dhs, dx=dxs, fwd_elems=fwd_elems, bwd_elems=bwd_elems)
