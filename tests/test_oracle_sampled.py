"""The row-at-a-time oracle (oracle/sampled.py, used for full-size checks) must agree with the step-by-step
oracle on small graphs, where both can be run in full."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import layer as olayer
from oracle import mask as omask
from oracle import partition as opart
from oracle import sampled as osamp
from paper_2406_17611_amd import synth

KEY = 0x240617611


@pytest.mark.parametrize("conv", ["gcn", "sage"])
def test_sampled_rows_match_full_oracle(conv):
    g = synth.small_random_graph(400, 7.0, conv, seed=3)
    n_parts, fi, fo, k, step, layer = 3, 20, 12, 5, 6, 1
    part = synth.random_partition(g.n, n_parts, seed=4)
    parts = opart.build_partitions(g.n, g.rowptr, g.colidx, g.vals, part, n_parts)
    rng = np.random.default_rng(5)
    x = rng.standard_normal((g.n, fi))
    h1 = rng.standard_normal((fi, fo)) * 0.3
    h0 = rng.standard_normal((fi, fo)) * 0.3 if conv == "sage" else None
    dxo = rng.standard_normal((g.n, fo))
    # full step-by-step oracle, one layer
    z_all = np.vstack([olayer.compress(x[p.local_gid], p.boundary_rows,
                                       omask.kept_columns(p.local_gid[p.boundary_rows], fi, k, KEY, step, layer))
                       for p in parts])
    m_full, xo_full = np.empty((g.n, fi)), np.empty((g.n, fo))
    for p in parts:
        cols = omask.kept_columns(p.halo_gid, fi, k, KEY, step, layer)
        xo, m = olayer.layer_forward(p, x[p.local_gid], z_all, cols, h1, h0, olayer.RELU)
        m_full[p.local_gid], xo_full[p.local_gid] = m, xo
    dx_full = np.zeros((g.n, fi))
    returned = {}
    for p in parts:
        cols = omask.kept_columns(p.halo_gid, fi, k, KEY, step, layer)
        _, _, dxl, dzh = olayer.layer_backward(p, dxo[p.local_gid], xo_full[p.local_gid], x[p.local_gid],
                                               m_full[p.local_gid], cols, h1, h0, olayer.RELU, True)
        dx_full[p.local_gid] += dxl
        returned[p.q] = (p.halo_gid, dzh)
        for o in range(n_parts):
            s0, s1 = p.halo_owner_ptr[o], p.halo_owner_ptr[o + 1]
            rows = parts[o].local_gid[parts[o].boundary_rows[p.halo_src_row[s0:s1]]]
            olayer.scatter_add(dx_full, rows, cols[s0:s1], dzh[s0:s1])
    # row-at-a-time oracle on a sample
    nodes = rng.permutation(g.n)[:60]
    m_s, xo_s = osamp.forward_rows(g.rowptr, g.colidx, g.vals, part, x, nodes, k, KEY, step, layer, h1, h0, True)
    assert np.allclose(m_s, m_full[nodes], rtol=1e-12, atol=1e-12)
    assert np.allclose(xo_s, xo_full[nodes], rtol=1e-12, atol=1e-12)
    st = sp.csr_matrix((g.vals.astype(np.float64), g.colidx, g.rowptr), shape=(g.n, g.n)).T.tocsr()
    st.sort_indices()
    dx_s = osamp.backward_rows(st.indptr, st.indices, st.data, part, dxo, xo_full, nodes, k, KEY, step, layer, h1, h0, True)
    assert np.allclose(dx_s, dx_full[nodes], rtol=1e-11, atol=1e-12)
    for q in range(n_parts):
        gids, dzh = returned[q]
        pick = np.arange(0, len(gids), 7)
        r = osamp.returned_rows(st.indptr, st.indices, st.data, part, dxo, xo_full, q, gids[pick], k, KEY, step,
                                layer, h1, True)
        assert np.allclose(r, dzh[pick], rtol=1e-11, atol=1e-12)
