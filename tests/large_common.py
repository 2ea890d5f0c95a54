"""Full-size GPU parity checks shared by the large configurations, in the launch configuration bench.py
times. The whole oracle cannot run at these sizes in seconds, so every layer is fed seeded synthetic inputs
(never outputs of the device path) and checked on sampled rows that the row-at-a-time oracle computes from
their definition on the global graph, on weight gradients (dense fp64 products), on exact exchange counts,
and on the index structures of one partition against the oracle's builder."""
import numpy as np
import scipy.sparse as sp
import torch

from gpu_common import KEY, assert_close
from oracle import mask as omask
from oracle import partition as opart
from oracle import sampled as osamp
from paper_2406_17611_amd import binding as vb
from paper_2406_17611_amd import synth
from paper_2406_17611_amd.runner import PartitionedNetwork

N_SAMPLE = 48


def build_large(workload):
    w = synth.make_workload(workload)
    g = w.graph
    host = vb.partition_build(g.n, g.rowptr, g.colidx, g.vals, w.part, w.n_parts)
    net = PartitionedNetwork(host, w.widths, w.conv, KEY, dtype=w.dtype)
    L = len(w.widths) - 1
    h1 = [synth.glorot(w.widths[l], w.widths[l + 1], synth.SEED_WEIGHT, 2 * l) for l in range(L)]
    h0 = [synth.glorot(w.widths[l], w.widths[l + 1], synth.SEED_WEIGHT, 2 * l + 1) for l in range(L)] \
        if w.conv == "sage" else None
    net.set_weights(h1, h0)
    order = np.concatenate([hp.local_gid for hp in host]).astype(np.int64)   # arena row -> global id
    st = sp.csr_matrix((g.vals, g.colidx, g.rowptr), shape=(g.n, g.n)).T.tocsr()
    st.sort_indices()
    return dict(w=w, g=g, host=host, net=net, h1=h1, h0=h0, order=order, st=st)


def stored(a, dtype):
    """The values both sides start from: fp32 as drawn, or their nearest bf16 values (input preparation)."""
    if dtype == "bf16":
        return torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    return a


def _to_arena(t, global_array, order):
    t.copy_(torch.from_numpy(np.ascontiguousarray(global_array[order])))


def check_partition_indexing(large, q):
    w, g, host = large["w"], large["g"], large["host"]
    op = opart.build_partitions(g.n, g.rowptr, g.colidx, g.vals, w.part, w.n_parts, only=[q])[0]
    hp = host[q]
    assert (hp.n_local, hp.n_halo, hp.n_boundary, hp.z_row_offset, hp.nnz) == \
           (op.n_local, op.n_halo, op.n_boundary, op.z_row_offset, op.nnz)
    for name in ("rowptr", "colidx", "vals", "t_rowptr", "t_colidx", "t_vals", "local_gid", "halo_gid",
                 "halo_owner_ptr", "boundary_rows", "halo_src_row", "halo_zrow"):
        assert np.array_equal(getattr(hp, name), getattr(op, name)), name


def check_layer(large, layer, ratio, tol, dh_cols=None, consumer=5, transform_first=False):
    """Forward then backward of one layer over all partitions on synthetic inputs; `dh_cols`: check that many
    sampled columns of the weight gradients instead of all of them. transform_first: the device forms S (X H)
    instead of (S X) H (same oracle); its weight gradient then depends on the true aggregates, which the oracle
    has for the sampled rows only, so it is checked in a second backward pass whose upstream gradient is zero
    outside those rows."""
    ctx = large["net"].ctx
    if not transform_first:
        return _check_layer(large, layer, ratio, tol, dh_cols, consumer, False)
    ctx.begin_step(0)
    ctx.set_layer_order(layer, vb.ORDER_TRANSFORM_FIRST)
    try:
        return _check_layer(large, layer, ratio, tol, dh_cols, consumer, True)
    finally:
        ctx.begin_step(1)
        ctx.set_layer_order(layer, vb.ORDER_AGGREGATE_FIRST)


def _check_layer(large, layer, ratio, tol, dh_cols, consumer, transform_first):
    w, g, host, net, order, st = (large[k] for k in ("w", "g", "host", "net", "order", "st"))
    part = w.part
    L = net.L
    sage = w.conv == "sage"
    fi, fo = w.widths[layer], w.widths[layer + 1]
    relu = layer < L - 1
    step = 10 + layer
    h1 = large["h1"][layer]
    h0 = large["h0"][layer] if sage else None
    k = omask.keep_count(fi, *ratio)

    # ---- forward: synthetic layer input for every node
    x = stored(synth.features(g.n, fi, synth.SEED_FEAT + 10 * layer), w.dtype)
    _to_arena(net.x[layer], x, order)
    ctx = net.ctx
    ctx.begin_step(step)
    ctx.set_ratio(-1, *ratio)
    assert ctx.keep(layer) == k
    net._ensure_buffers()
    ctx.reset_stats()
    for p, hp in enumerate(host):
        ctx.compress(layer, net.boundary_gid[p], net.dev_parts[p]["boundary_rows"], hp.n_boundary,
                     net.x[layer][net.rows(p)], fi, net.z[layer][hp.z_row_offset * k:])
    for q in range(net.P):
        r = net.rows(q)
        ctx.layer_fwd(layer, q, net.x[layer][r], net.z[layer], net.h1[layer], net.h0[layer], net.x[layer + 1][r],
                      None, net.m[layer][r])
    torch.cuda.synchronize()
    halo_rows = sum(h.n_halo for h in host)
    assert ctx.stats()["fwd_elems"][layer] == halo_rows * k          # compressed rows x k, exactly

    rng = np.random.default_rng(100 + layer)
    deg = np.diff(g.rowptr)
    hubs = np.argsort(deg)[-3:]                                       # the longest rows (split across wavefronts)
    nodes = np.unique(np.concatenate([rng.integers(0, g.n, size=N_SAMPLE), hubs]))
    arena_of = np.empty(g.n, dtype=np.int64)
    arena_of[order] = np.arange(g.n)
    m_ref, xo_ref = osamp.forward_rows(g.rowptr, g.colidx, g.vals, part, x, nodes, k, KEY, step, layer, h1, h0, relu)
    rows_dev = torch.from_numpy(arena_of[nodes]).cuda()
    if not transform_first:
        assert_close(net.m[layer][rows_dev].float().cpu().numpy(), m_ref, f"layer {layer} M rows", tol)
    assert_close(net.x[layer + 1][rows_dev].float().cpu().numpy(), xo_ref, f"layer {layer} X_out rows", tol)
    # compressed boundary rows are copies: bit-exact on a sample of owners' rows
    for p in (0, net.P - 1):
        hp = host[p]
        pick = rng.integers(0, hp.n_boundary, size=200)
        gids = hp.local_gid[hp.boundary_rows[pick]]
        cols = omask.kept_columns(gids, fi, k, KEY, step, layer)
        z = net.z[layer][:net.b_total * k].reshape(net.b_total, k)[torch.from_numpy(hp.z_row_offset + pick).cuda()]
        assert np.array_equal(z.float().cpu().numpy(), x[gids[:, None], cols])

    # ---- backward: synthetic upstream gradient, stored activations and aggregates
    dxo = stored(synth.upstream_grad(g.n, fo, synth.SEED_GRAD + layer) * np.float32(g.n), w.dtype)
    xout = stored(synth.features(g.n, fo, synth.SEED_FEAT + 10 * layer + 1), w.dtype)   # sign pattern of the ReLU gate
    msav = stored(synth.features(g.n, fi, synth.SEED_FEAT + 10 * layer + 2), w.dtype)
    _to_arena(net.dx[layer + 1], dxo, order)
    _to_arena(net.x[layer + 1], xout, order)
    _to_arena(net.m[layer], msav, order)
    net.zero_grads()
    need = layer > 0
    for q in range(net.P):
        r = net.rows(q)
        dzh = net.dz_halo[layer][int(net.halo_off[q]) * k:] if need else None
        ctx.layer_bwd(layer, q, net.dx[layer + 1][r], net.x[layer + 1][r], net.x[layer][r],
                      net.z[layer] if transform_first else net.m[layer][r],
                      net.h1[layer], net.h0[layer], net.dh1[layer], net.dh0[layer],
                      net.dx[layer][r] if need else None, dzh)
    if need:
        for p in range(net.P):
            ctx.accumulate_returned(layer, p, net.ret_ptr[p], net.ret_src[p], net.dz_halo[layer],
                                    net.dx[layer][net.rows(p)])
    torch.cuda.synchronize()
    assert ctx.stats()["bwd_elems"][layer] == (halo_rows * k if need else 0)

    # weight gradients are fp32 sums over all nodes (no storage rounding): fp32 bound for either storage type
    cols = np.arange(fo) if dh_cols is None or dh_cols >= fo else np.sort(rng.choice(fo, size=dh_cols, replace=False))
    dz = dxo[:, cols].astype(np.float64)
    if relu:
        dz *= xout[:, cols] > 0
    if not transform_first:
        assert_close(net.dh1[layer].cpu().numpy()[:, cols], msav.astype(np.float64).T @ dz, f"layer {layer} dH1")
    if sage:
        assert_close(net.dh0[layer].cpu().numpy()[:, cols], x.astype(np.float64).T @ dz, f"layer {layer} dH0")
    del dz
    if need:
        dx_ref = osamp.backward_rows(st.indptr, st.indices, st.data, part, dxo, xout, nodes, k, KEY, step, layer,
                                     h1, h0, relu)
        assert_close(net.dx[layer][rows_dev].float().cpu().numpy(), dx_ref, f"layer {layer} dX rows", tol)
        q = consumer
        hp = host[q]
        pick = np.unique(np.concatenate([rng.integers(0, hp.n_halo, size=N_SAMPLE),
                                         np.argsort(np.diff(hp.t_rowptr)[hp.n_local:])[-2:]]))
        ret_ref = osamp.returned_rows(st.indptr, st.indices, st.data, part, dxo, xout, q, hp.halo_gid[pick], k, KEY,
                                      step, layer, h1, relu)
        got = net.dz_halo[layer][int(net.halo_off[q]) * k:int(net.halo_off[q + 1]) * k].reshape(hp.n_halo, k)
        assert_close(got[torch.from_numpy(pick).cuda()].float().cpu().numpy(), ret_ref,
                     f"layer {layer} returned rows", tol)
    if transform_first:
        # weight gradient of the aggregated tap: upstream gradient on the sampled rows only, whose aggregates the
        # oracle computed above (the layer has no gate: transform-first is limited to identity activations)
        assert not relu
        sparse = np.zeros_like(dxo)
        sparse[nodes] = dxo[nodes]
        _to_arena(net.dx[layer + 1], sparse, order)
        net.zero_grads()
        for q in range(net.P):
            r = net.rows(q)
            ctx.layer_bwd(layer, q, net.dx[layer + 1][r], net.x[layer + 1][r], net.x[layer][r], net.z[layer],
                          net.h1[layer], net.h0[layer], net.dh1[layer], net.dh0[layer], None, None)
        torch.cuda.synchronize()
        assert_close(net.dh1[layer].cpu().numpy(), m_ref.astype(np.float64).T @ dxo[nodes].astype(np.float64),
                     f"layer {layer} dH1 from the sampled rows", tol)
