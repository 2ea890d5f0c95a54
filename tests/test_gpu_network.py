"""GPU parity of the whole path (all layers, all partitions in turn, forward and backward, exchange
hand-offs and owner-side accumulation) on the benchmark configurations the oracle finishes in seconds."""
import numpy as np
import pytest
import torch

from gpu_common import KEY, assert_close, both_partitions
from oracle import layer as olayer
from oracle import mask as omask
from oracle.rounding import round_bf16
from paper_2406_17611_amd import synth
from paper_2406_17611_amd.runner import PartitionedNetwork

pytestmark = pytest.mark.gpu

# Norm-wise bound of the chained bf16 configuration. Every bf16 rounding is within 2^-9 relative, and up to six of
# them lie between the (bf16-exact) inputs and a gradient dX_l: the bf16 copy of the weights fed to the matrix
# cores, the stored dM, the compressed rows handed back, and three stores of dX_l (transposed aggregation, self
# tap, owner-side sum); the oracle rounds at the stores only. 6 * 2^-9 < 2^-6.
BF16_TOL = 2.0 ** -6


def _weights(widths, conv):
    h1 = [synth.glorot(widths[l], widths[l + 1], synth.SEED_WEIGHT, 2 * l) for l in range(len(widths) - 1)]
    h0 = [synth.glorot(widths[l], widths[l + 1], synth.SEED_WEIGHT, 2 * l + 1) for l in range(len(widths) - 1)] \
        if conv == "sage" else None
    return h1, h0


def _f32(a):
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


def _compare_network(g, part, n_parts, conv, widths, ratios, steps, tol=1e-4, dtype="f32", n_streams=1, transform_first=()):
    """dtype "bf16": inputs are bf16 values, the oracle rounds to bf16 where the device stores bf16
    (activations, aggregates, messages, gradients) and `tol` is the bound of that configuration.
    transform_first: layers the device runs as S (X H) instead of (S X) H; the oracle is the same (the products
    associate), only the aggregated rows M of those layers do not exist on the device."""
    host, orc = both_partitions(g, part, n_parts)
    L = len(widths) - 1
    x0 = synth.features(g.n, widths[0], synth.SEED_FEAT)
    dxl = synth.upstream_grad(g.n, widths[-1], synth.SEED_GRAD)
    stored = _f32
    if dtype == "bf16":
        stored = round_bf16
        x0, dxl = round_bf16(x0).astype(np.float32), round_bf16(dxl).astype(np.float32)
    h1, h0 = _weights(widths, conv)
    net = PartitionedNetwork(host, widths, conv, KEY, dtype=dtype, n_streams=n_streams, transform_first=transform_first)
    net.set_inputs(x0)
    net.set_weights(h1, h0)
    net.set_upstream(dxl)
    acts = [olayer.RELU] * (L - 1) + [olayer.IDENTITY]
    weights = [(h1[l], h0[l] if h0 is not None else None) for l in range(L)]
    op_norm = _aggregation_norm_bound(g, part)
    total_flips = 0
    for step, ratio in zip(steps, ratios):
        net.zero_grads()
        net.ctx.reset_stats()
        net.forward(step, ratio)
        torch.cuda.synchronize()
        per_layer = ratio if isinstance(ratio[0], (tuple, list)) else [ratio] * L
        keep = [omask.keep_count(widths[l], *per_layer[l]) for l in range(L)]
        assert [net.ctx.keep(l) for l in range(L)] == keep
        ref = olayer.network_step(orc, [x0[p.local_gid] for p in orc], weights, acts, keep, KEY, step,
                                  [dxl[p.local_gid] for p in orc], round_store=stored)
        tag = f"step {step} ratio {ratio}"
        assert net.ctx.stats()["fwd_elems"] == ref["fwd_elems"], tag
        # forward: free-running chain on both sides
        for l in range(L):
            assert_close(net.to_global(net.x[l + 1]), _gather(orc, ref["x"][l + 1], g.n), f"{tag} X_{l + 1}", tol)
            if l not in transform_first:
                assert_close(net.to_global(net.m[l]), _gather(orc, ref["m"][l], g.n), f"{tag} M_{l}", tol)
            k = keep[l]
            z = net.z[l][:net.b_total * k].reshape(net.b_total, k).float().cpu().numpy()
            if l == 0:
                assert np.array_equal(z, ref["z"][0].astype(np.float32)), f"{tag} Z_0 must be bit-exact"
            else:
                assert_close(z, ref["z"][l], f"{tag} Z_{l}", tol)
        # backward, first pass: free-running on the device's own saved activations and aggregates
        flips = _check_free_running_backward(net, orc, ref, g.n, conv, weights, acts, op_norm, tol, tag)
        assert net.ctx.stats()["bwd_elems"] == ref["bwd_elems"], tag
        total_flips += sum(flips)
        print(f"[free-running backward] {tag}: gate elements decided the other way per layer {flips}")
        net.zero_grads()
        # backward, second pass: the ReLU gate [x_out > 0] is a discrete decision, and a single element decided
        # the other way moves the gradients by far more than the parity bound. Here both sides take it on the
        # same stored activations: the oracle's stored activations and aggregates become the saved tensors
        # of the device path (oracle -> device); the gradient chain itself (dX through all layers, returned errors,
        # owner-side accumulation, weight-gradient sums) then runs free on the device and must meet the plain bound.
        for l in range(L + 1):
            net.x[l].copy_(torch.from_numpy(np.vstack(ref["x"][l]).astype(np.float32)))
        for l in range(L):
            net.m[l].copy_(torch.from_numpy(np.vstack(ref["m"][l]).astype(np.float32)))
        net.backward()
        torch.cuda.synchronize()
        for l in range(L):
            assert_close(net.dh1[l].cpu().numpy(), ref["dh"][l][0], f"{tag} dH1_{l}", tol)
            if conv == "sage":
                assert_close(net.dh0[l].cpu().numpy(), ref["dh"][l][1], f"{tag} dH0_{l}", tol)
        for l in range(1, L):
            assert_close(net.to_global(net.dx[l]), _gather(orc, ref["dx"][l], g.n), f"{tag} dX_{l}", tol)
        assert net.ctx.stats()["bwd_elems"] == [2 * e for e in ref["bwd_elems"]], tag      # two backward passes
    net.total_gate_flips = total_flips
    return net


def _spectral_norm(a):
    """Largest singular value of a sparse matrix (power iteration on a^T a by the library routine), with 1 %
    of head-room for the iteration's own error."""
    from scipy.sparse.linalg import svds
    if a.nnz == 0:
        return 0.0
    if min(a.shape) <= 2:
        return float(np.linalg.norm(a.toarray(), 2))
    return 1.01 * float(svds(a.astype(np.float64), k=1, return_singular_vectors=False, tol=1e-6)[0])


def _aggregation_norm_bound(g, part):
    """Bound on ||dX||_F / ||dM||_F of the transposed aggregation with the compressed hand-back: dX = S_intra^T dM
    + Mask * (S_cross^T dM), and an element-wise 0/1 mask never increases a Frobenius norm, so the ratio is at
    most ||S_intra||_2 + ||S_cross||_2."""
    import scipy.sparse as sp
    s = sp.csr_matrix((g.vals, g.colidx, g.rowptr), shape=(g.n, g.n)).tocoo()
    same = part[s.row] == part[s.col]
    intra = sp.csr_matrix((s.data[same], (s.row[same], s.col[same])), shape=s.shape)
    cross = sp.csr_matrix((s.data[~same], (s.row[~same], s.col[~same])), shape=s.shape)
    return _spectral_norm(intra) + _spectral_norm(cross)


def _check_free_running_backward(net, orc, ref, n, conv, weights, acts, op_norm, tol, tag):
    """Runs the device's backward pass on the device's own forward results and compares it with the oracle's own
    chain. The two chains differ (beyond rounding, which `tol` covers) only through ReLU gate decisions taken the
    other way, which can happen only where the argument of the nonlinearity is within the parity bound of zero:

      * every element whose gate differs must have |Zpre_ref| <= tol * ||Zpre_ref||_inf;
      * the gradients may deviate by tol (norm-wise, as everywhere) plus what those elements can cause, bounded
        from the oracle's tensors. With D_l the differing elements of layer l, delta_l a bound on the Frobenius
        norm of the deviation of dX_l (delta_L = 0) and dZ = dX * gate:
            ||dZ_dev - dZ_ref||_F <= delta_{l+1} + f_l,              f_l = || dX_ref restricted to D_l ||_F
            ||dH1_dev - dH1_ref||_F <= sum_{(i,c) in D_l} |dX_ref[i,c]| ||M_ref[i,:]||_2 + ||M_ref||_2 delta_{l+1}
            (dH0: X_{l-1} in place of M)
            delta_l = (op_norm ||H1||_2 + ||H0||_2) (delta_{l+1} + f_l)
      * columns of the topmost gated layer's weight gradients that hold no differing element see no deviation at
        all (the layer above has no gate) and must meet the plain bound.
    Returns the number of differing gate elements per layer."""
    L = net.L
    net.backward()
    torch.cuda.synchronize()
    flips = [0] * L
    delta = 0.0                                   # deviation of dX_{l+1}
    for l in range(L - 1, -1, -1):
        dx_up = _gather(orc, ref["dx"][l + 1], n)
        dev_out = net.to_global(net.x[l + 1])
        f_l, dh_flip = 0.0, [0.0, 0.0]
        clean_cols = np.ones(dx_up.shape[1], dtype=bool)
        if acts[l] == olayer.RELU:
            zpre = _gather(orc, ref["zpre"][l], n)
            differs = (dev_out > 0) != (_gather(orc, ref["x"][l + 1], n) > 0)
            rows, cols = np.nonzero(differs)
            flips[l] = rows.shape[0]
            if flips[l]:
                band = tol * np.abs(zpre).max()
                assert np.abs(zpre[rows, cols]).max() <= band, \
                    f"{tag}: gate of layer {l} differs where |Zpre| = {np.abs(zpre[rows, cols]).max():.3e} > {band:.3e}"
                in_band = int((np.abs(zpre) <= band).sum())
                assert flips[l] <= in_band
                mag = np.abs(dx_up[rows, cols])
                f_l = float(np.linalg.norm(mag))
                dh_flip[0] = float(mag @ np.linalg.norm(_gather(orc, ref["m"][l], n)[rows], axis=1))
                dh_flip[1] = float(mag @ np.linalg.norm(_gather(orc, ref["x"][l], n)[rows], axis=1))
                clean_cols[np.unique(cols)] = False
        pairs = [(net.dh1[l], ref["dh"][l][0], ref["m"][l], dh_flip[0], "dH1")]
        if conv == "sage":
            pairs.append((net.dh0[l], ref["dh"][l][1], ref["x"][l], dh_flip[1], "dH0"))
        for got, want, left, flip_part, name in pairs:
            left_norm = float(np.linalg.norm(np.vstack(left), 2)) if delta > 0 else 0.0
            _assert_close_plus(got.cpu().numpy(), want, tol, flip_part + left_norm * delta, f"{tag} free-running {name}_{l}")
            if delta == 0.0 and clean_cols.any():
                assert_close(got.cpu().numpy()[:, clean_cols], want[:, clean_cols],
                             f"{tag} free-running {name}_{l}, columns without a differing gate", tol)
        if l == 0:
            break
        h1, h0 = weights[l]
        gain = op_norm * np.linalg.norm(h1, 2) + (np.linalg.norm(h0, 2) if h0 is not None else 0.0)
        delta = float(gain * (delta + f_l))
        _assert_close_plus(net.to_global(net.dx[l]), _gather(orc, ref["dx"][l], n), tol, delta,
                           f"{tag} free-running dX_{l}")
    return flips


def _assert_close_plus(got, ref, tol, extra, what):
    """assert_close with an additive allowance `extra` (a bound on the Frobenius norm, hence also on the largest
    element, of a deviation that is not rounding)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    diff = got - ref
    inf_err, fro_err = np.abs(diff).max(initial=0.0), np.linalg.norm(diff)
    assert inf_err <= tol * np.abs(ref).max(initial=0.0) + extra + 1e-30, f"{what}: max err {inf_err:.3e}, allowance {extra:.3e}"
    assert fro_err <= tol * np.linalg.norm(ref) + extra + 1e-30, f"{what}: fro err {fro_err:.3e}, allowance {extra:.3e}"


def _gather(parts, per_part, n):
    out = np.empty((n, per_part[0].shape[1]))
    for p in parts:
        out[p.local_gid] = per_part[p.q]
    return out


def test_tiny_config_full_step():
    w = synth.make_workload("tiny")
    _compare_network(w.graph, w.part, w.n_parts, w.conv, w.widths, [(4, 1), (1, 1)], steps=[0, 1])


def test_medium_config_all_ratios():
    w = synth.make_workload("medium")
    _compare_network(w.graph, w.part, w.n_parts, w.conv, w.widths, list(w.ratios), steps=list(range(len(w.ratios))))


def test_medium_bfs16_config_on_the_variable_schedule():
    w = synth.make_workload("medium_bfs16")
    steps = [0, 1, 50, 98, 99]
    _compare_network(w.graph, w.part, w.n_parts, w.conv, w.widths, [w.ratios[t] for t in steps], steps=steps)


def test_sage_network_small():
    g = synth.small_random_graph(3000, 10.0, "sage", seed=31)
    part = synth.random_partition(g.n, 4, seed=32)
    _compare_network(g, part, 4, "sage", (100, 256, 256, 47), [(8, 1), (2, 1)], steps=[5, 6])


@pytest.mark.parametrize("n_streams", [2, 3])
def test_partitions_dealt_to_several_streams(n_streams):
    # overlapping layer calls on different streams (per-stream workspaces, joins at layer boundaries and before
    # the owner-side sums, per-stream weight-gradient accumulators folded at the end) give the oracle's results
    g = synth.small_random_graph(3000, 10.0, "sage", seed=31)
    part = synth.random_partition(g.n, 5, seed=32)
    _compare_network(g, part, 5, "sage", (100, 256, 256, 47), [(8, 1), (1, 1)], steps=[5, 6], n_streams=n_streams)
    w = synth.make_workload("medium")
    _compare_network(w.graph, w.part, w.n_parts, w.conv, w.widths, [(8, 1)], steps=[3], n_streams=n_streams)


@pytest.mark.parametrize("conv,dtype", [("gcn", "f32"), ("sage", "f32"), ("gcn", "bf16")])
def test_no_communication_and_no_intermediate_communication(conv, dtype):
    # unbounded ratio (k = 0) on every layer, then only on the layers after the first (input features of adjacent
    # nodes still exchanged, at ratio 2): remote nodes contribute nothing there, forward or backward
    g = synth.small_random_graph(2500, 9.0, conv, seed=61)
    part = synth.random_partition(g.n, 3, seed=62)
    tol = BF16_TOL if dtype == "bf16" else 1e-4
    net = _compare_network(g, part, 3, conv, (64, 128, 128, 10), [(1, 0), [(2, 1), (1, 0), (1, 0)]], steps=[1, 2],
                           tol=tol, dtype=dtype)
    st = net.ctx.stats()
    assert st["fwd_elems"][1:] == [0, 0] and st["bwd_elems"] == [0, 0, 0] and st["fwd_elems"][0] > 0


def test_tiny_config_full_step_bf16_storage():
    w = synth.make_workload("tiny")
    _compare_network(w.graph, w.part, w.n_parts, w.conv, w.widths, [(4, 1), (1, 1)], steps=[0, 1], tol=BF16_TOL,
                     dtype="bf16")


@pytest.mark.parametrize("conv", ["gcn", "sage"])
def test_network_small_bf16_storage(conv):
    # the widths of the bf16 configuration (100 -> 512 -> 512 -> 47) at its three ratios, on a graph the
    # oracle finishes in seconds, with 4 partitions
    g = synth.small_random_graph(3000, 10.0, conv, seed=51)
    part = synth.random_partition(g.n, 4, seed=52)
    _compare_network(g, part, 4, conv, (100, 512, 512, 47), [(1, 1), (4, 1), (32, 1)], steps=[2, 3, 4], tol=BF16_TOL,
                     dtype="bf16")


@pytest.mark.parametrize("conv", ["gcn", "sage"])
def test_transform_before_aggregate_on_the_class_layer(conv):
    # eq. (2) with the products in the other order on the narrowing last layer (512 -> 47): local rows and the
    # k-sparse halo rows are transformed first and rows of 47 elements aggregated, forward and backward, while the
    # exchange stays the compressed one; at full communication, two compression ratios and none at all
    g = synth.small_random_graph(3000, 10.0, conv, seed=51)
    part = synth.random_partition(g.n, 4, seed=52)
    net = _compare_network(g, part, 4, conv, (100, 512, 512, 47), [(1, 1), (4, 1), (32, 1), (1, 0)], steps=[2, 3, 4, 5],
                           tol=BF16_TOL, dtype="bf16", transform_first=(2,))
    assert net.ctx.stats()["fwd_elems"][2] == 0          # the last step exchanged nothing


def test_two_runs_give_identical_bits():
    w = synth.make_workload("tiny")
    outs = []
    for _ in range(2):
        net = _compare_network(w.graph, w.part, w.n_parts, w.conv, w.widths, [(4, 1)], steps=[7])
        outs.append([t.cpu().numpy().copy() for t in net.x[1:] + net.dh1 + net.dx[1:]])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_owner_side_accumulation_matches_per_consumer_scatter():
    """varco_accumulate_returned against the oracle's per-consumer scatter-add on random returned rows."""
    from gpu_common import dev
    from oracle import partition as opart
    from paper_2406_17611_amd import binding as vb
    g = synth.small_random_graph(2500, 9.0, "gcn", seed=41)
    part = synth.random_partition(g.n, 5, seed=42)
    host, orc = both_partitions(g, part, 5)
    width, ratio, layer, step = 128, (8, 1), 1, 4
    net = PartitionedNetwork(host, (16, width, 8), "gcn", KEY)
    net.ctx.begin_step(step)
    net.ctx.set_ratio(layer, *ratio)
    k = net.ctx.keep(layer)
    rng = np.random.default_rng(0)
    returned = [rng.standard_normal((p.n_halo, k)).astype(np.float32) for p in orc]
    dx0 = rng.standard_normal((g.n, width)).astype(np.float32)
    want = [dx0[p.local_gid].astype(np.float64) for p in orc]
    for q, p in enumerate(orc):                      # oracle: consumers in ascending order
        cols = omask.kept_columns(p.halo_gid, width, k, KEY, step, layer)
        for o in range(5):
            s0, s1 = int(p.halo_owner_ptr[o]), int(p.halo_owner_ptr[o + 1])
            olayer.scatter_add(want[o], orc[o].boundary_rows[p.halo_src_row[s0:s1]], cols[s0:s1],
                               returned[q][s0:s1].astype(np.float64))
    ret_dev = dev(np.vstack(returned))
    for p_i, p in enumerate(orc):
        x = dev(dx0[p.local_gid])
        net.ctx.accumulate_returned(layer, p_i, net.ret_ptr[p_i], net.ret_src[p_i], ret_dev, x)
        assert_close(x.cpu().numpy(), want[p_i], f"owner {p_i}", 1e-6)
