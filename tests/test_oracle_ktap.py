"""Pins of the oracle's K-tap layer (eq. (1)-(2) with K > 2 and one compressed exchange per hop)."""
import numpy as np
import pytest

import dense_reference as dref
from oracle import ktap as oktap
from oracle import layer as olayer
from oracle import mask as omask
from oracle import partition as opart
from paper_2406_17611_amd import synth

KEY = 0x240617611


def _close(a, b, tol=1e-10):
    return np.abs(np.asarray(a) - np.asarray(b)).max() <= tol * max(1.0, np.abs(np.asarray(b)).max())


def _setup(n_taps, n_parts, widths, seed):
    g = synth.small_random_graph(120, 5.0, "sage", seed=seed)
    part = synth.random_partition(g.n, n_parts, seed + 1)
    parts = opart.build_partitions(g.n, g.rowptr, g.colidx, g.vals, part, n_parts)
    rng = np.random.default_rng(seed + 2)
    x = rng.standard_normal((g.n, widths[0]))
    weights = [[rng.standard_normal((widths[l], widths[l + 1])) * 0.4 for _ in range(n_taps)]
               for l in range(len(widths) - 1)]
    r = rng.standard_normal((g.n, widths[-1]))
    return g, part, parts, x, weights, r


def _gather(parts, per_part, n):
    out = np.empty((n, per_part[0].shape[1]))
    for p in parts:
        out[p.local_gid] = per_part[p.q]
    return out


def _dense(g, part, x, weights, r, keep, step):
    """Partition-free statement with global keep-masks: Y_k = S_intra Y_{k-1} + S_cross (Mask_k * Y_{k-1})."""
    s = dref.dense_operator(g)
    s_in, s_x = dref.split_operator(s, part)
    n_layers = len(weights)
    xs, yss, masks = [x], [], []
    for l, hs in enumerate(weights):
        ys, mk = [xs[l]], [None]
        for hop in range(1, len(hs)):
            m = omask.keep_mask(np.arange(g.n), xs[l].shape[1], keep[l], KEY, step, oktap.tap(l, hop))
            ys.append(s_in @ ys[-1] + s_x @ (m * ys[-1]))
            mk.append(m)
        zpre = sum(y @ h for y, h in zip(ys, hs))
        xs.append(np.maximum(zpre, 0.0) if l < n_layers - 1 else zpre)
        yss.append(ys), masks.append(mk)
    dhs, dxs, dx = [None] * n_layers, {}, r
    for l in range(n_layers - 1, -1, -1):
        hs = weights[l]
        dz = dx * (xs[l + 1] > 0) if l < n_layers - 1 else dx
        dhs[l] = [yss[l][hop].T @ dz for hop in range(len(hs))]
        if l == 0:
            break
        gk = dz @ hs[-1].T
        for hop in range(len(hs) - 1, 0, -1):
            gk = dz @ hs[hop - 1].T + s_in.T @ gk + masks[l][hop] * (s_x.T @ gk)
        dx = gk
        dxs[l] = dx
    return xs, yss, dhs, dxs


@pytest.mark.parametrize("n_taps,n_parts,ratio", [(3, 2, 1), (3, 3, 2), (4, 4, 4), (2, 3, 2)])
def test_ktap_equals_dense_statement(n_taps, n_parts, ratio):
    widths = (12, 16, 6)
    g, part, parts, x, weights, r = _setup(n_taps, n_parts, widths, seed=20 + n_taps)
    keep = [omask.keep_count(w, ratio, 1) for w in widths[:-1]]
    acts = [olayer.RELU, olayer.IDENTITY]
    res = oktap.network_step(parts, [x[p.local_gid] for p in parts], weights, acts, keep, KEY, 3,
                             [r[p.local_gid] for p in parts])
    xs, yss, dhs, dxs = _dense(g, part, x, weights, r, keep, 3)
    for l in range(2):
        assert _close(_gather(parts, res["x"][l + 1], g.n), xs[l + 1])
        for hop in range(n_taps):
            assert _close(_gather(parts, res["y"][l][hop], g.n), yss[l][hop])
            assert _close(res["dh"][l][hop], dhs[l][hop])
    assert _close(_gather(parts, res["dx"][1], g.n), dxs[1])
    halo_rows = sum(p.n_halo for p in parts)
    assert res["fwd_elems"] == [halo_rows * k * (n_taps - 1) for k in keep]
    assert res["bwd_elems"] == [0, halo_rows * keep[1] * (n_taps - 1)]
    if ratio == 1:      # lossless: eq. (2) on the unpartitioned graph, powers of the dense operator
        s = dref.dense_operator(g)
        zpre = sum(np.linalg.matrix_power(s, hop) @ x @ weights[0][hop] for hop in range(n_taps))
        assert _close(_gather(parts, res["x"][1], g.n), np.maximum(zpre, 0.0))


def test_two_taps_are_the_sage_layer():
    widths = (10, 14, 5)
    g, part, parts, x, weights, r = _setup(2, 3, widths, seed=33)
    keep = [omask.keep_count(w, 2, 1) for w in widths[:-1]]
    acts = [olayer.RELU, olayer.IDENTITY]
    # hop 1 of the K-tap layer draws the positions of "layer" l + 16, the two-tap layer those of l: compare at ratio 1
    keep1 = list(widths[:-1])
    a = oktap.network_step(parts, [x[p.local_gid] for p in parts], weights, acts, keep1, KEY, 0,
                           [r[p.local_gid] for p in parts])
    b = olayer.network_step(parts, [x[p.local_gid] for p in parts], [(w[1], w[0]) for w in weights], acts, keep1, KEY, 0,
                            [r[p.local_gid] for p in parts])
    for l in range(2):
        assert _close(_gather(parts, a["x"][l + 1], g.n), _gather(parts, b["x"][l + 1], g.n))
        assert _close(a["dh"][l][1], b["dh"][l][0]) and _close(a["dh"][l][0], b["dh"][l][1])
    assert _close(_gather(parts, a["dx"][1], g.n), _gather(parts, b["dx"][1], g.n))
    assert keep != keep1


def test_ktap_gradient_by_finite_differences():
    widths = (8, 9, 4)
    g, part, parts, x, weights, r = _setup(3, 3, widths, seed=41)
    keep = [4, 5]
    acts = [olayer.RELU, olayer.IDENTITY]
    x0 = [x[p.local_gid] for p in parts]
    rr = [r[p.local_gid] for p in parts]
    res = oktap.network_step(parts, x0, weights, acts, keep, KEY, 2, rr)

    def objective(ws):
        out = oktap.network_step(parts, x0, ws, acts, keep, KEY, 2, rr)
        return sum((out["x"][-1][p.q] * rr[p.q]).sum() for p in parts)

    rng = np.random.default_rng(0)
    eps = 1e-6
    for l in range(2):
        for hop in range(3):
            for _ in range(3):
                i, j = rng.integers(0, widths[l]), rng.integers(0, widths[l + 1])
                wp = [[h.copy() for h in hs] for hs in weights]
                wm = [[h.copy() for h in hs] for hs in weights]
                wp[l][hop][i, j] += eps
                wm[l][hop][i, j] -= eps
                fd = (objective(wp) - objective(wm)) / (2 * eps)
                assert abs(fd - res["dh"][l][hop][i, j]) <= 1e-6 * max(1.0, abs(fd))
