"""GPU parity of one partition's layer forward and backward (Algorithm 1 for one layer of eq. (2)) against
the CPU oracle, on the same seeded inputs, through the C ABI."""
import numpy as np
import pytest
import torch

from gpu_common import KEY, TOL, assert_close, both_partitions, dev, hub_graph
from oracle import layer as olayer
from oracle import mask as omask
from oracle.rounding import round_bf16
from paper_2406_17611_amd import binding as vb
from paper_2406_17611_amd import synth

pytestmark = pytest.mark.gpu


BF16_TOL = 2.0 ** -7   # norm-wise bound with bf16 storage: at most four roundings of 2^-9 (weight copy, dM, two stores)


def _run_layer_case(g, part, n_parts, conv, fi, fo, ratio, act, seed, step=3, layer=1, dtype="f32", z_row_shift=0,
                    registered_before=None, transform_first=False):
    """dtype "bf16": every activation / message / gradient tensor handed to the library is bf16 (the inputs
    are bf16 values, so both sides start from identical numbers); weights and weight gradients stay fp32.
    z_row_shift: the library's partitions address the compressed buffer that many rows further in (the rows
    before stay unused), the oracle's are unchanged. registered_before: partitions of another graph that are
    registered under the same numbers first, and replaced. transform_first: the layer runs as S (X H) (same oracle;
    no aggregated rows M on the device, the backward call is given the compressed buffer again)."""
    host, orc = both_partitions(g, part, n_parts)
    for hp in host:
        hp.halo_zrow = (hp.halo_zrow.astype(np.int64) + z_row_shift).astype(np.int32)
        hp.z_row_offset += z_row_shift
    rng = np.random.default_rng(seed)
    sage = conv == "sage"
    widths = [8, fi, fo]
    bf16 = dtype == "bf16"
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = BF16_TOL if bf16 else TOL
    stored = (lambda a: round_bf16(a).astype(np.float32)) if bf16 else (lambda a: np.asarray(a, dtype=np.float32))
    ctx = vb.Context(widths, [vb.ACT_RELU, act], vb.CONV_SAGE if sage else vb.CONV_GCN, n_parts, KEY,
                     vb.BF16 if bf16 else vb.F32)
    for q, hp in enumerate(registered_before or []):
        ctx.register_partition(q, hp)
    for q, hp in enumerate(host):
        ctx.register_partition(q, hp)
    ctx.prepare()
    ctx.begin_step(step)
    ctx.set_ratio(layer, *ratio)
    if transform_first:
        ctx.set_layer_order(layer, vb.ORDER_TRANSFORM_FIRST)
    k = ctx.keep(layer)
    assert k == omask.keep_count(fi, *ratio)

    x = stored(rng.standard_normal((g.n, fi)))
    h1 = (rng.standard_normal((fi, fo)) * 0.3).astype(np.float32)
    h0 = (rng.standard_normal((fi, fo)) * 0.3).astype(np.float32) if sage else None
    dxo = stored(rng.standard_normal((g.n, fo)) / g.n)
    b_total = sum(p.n_boundary for p in orc)

    # owners' compressed boundary rows: oracle version, and the library's own through varco_compress
    z_ref = np.vstack([olayer.compress(x[p.local_gid], p.boundary_rows,
                                       omask.kept_columns(p.local_gid[p.boundary_rows], fi, k, KEY, step, layer))
                       for p in orc]) if b_total else np.zeros((0, k))
    z_dev = torch.empty((z_row_shift + max(b_total, 1), k), dtype=tdt, device="cuda")
    for q, p in enumerate(orc):
        if p.n_boundary:
            ctx.compress(layer, dev(p.local_gid[p.boundary_rows]), dev(p.boundary_rows), p.n_boundary,
                         dev(x[p.local_gid], tdt), fi, z_dev[z_row_shift + p.z_row_offset:])
    assert np.array_equal(z_dev[z_row_shift:z_row_shift + b_total].float().cpu().numpy(), z_ref.astype(np.float32))

    h1d, h0d = dev(h1), (dev(h0) if sage else None)
    dh1_dev = torch.zeros((fi, fo), dtype=torch.float32, device="cuda")
    dh0_dev = torch.zeros((fi, fo), dtype=torch.float32, device="cuda") if sage else None
    dh1_ref = np.zeros((fi, fo))
    dh0_ref = np.zeros((fi, fo))
    o_act = olayer.RELU if act == vb.ACT_RELU else olayer.IDENTITY
    halo_rows = 0
    for q, p in enumerate(orc):
        cols = omask.kept_columns(p.halo_gid, fi, k, KEY, step, layer)
        xl = x[p.local_gid]
        xo_ref, m_ref = olayer.layer_forward(p, xl, z_ref, cols, h1, h0, o_act)
        xld = dev(xl, tdt)
        xo = torch.full((p.n_local, fo), float("nan"), dtype=tdt, device="cuda")
        ms = torch.full((p.n_local, fi), float("nan"), dtype=tdt, device="cuda")
        ctx.layer_fwd(layer, q, xld, z_dev, h1d, h0d, xo, None, None if transform_first else ms)
        if not transform_first:
            assert_close(ms.float().cpu().numpy(), m_ref, f"M q={q}", tol)
        assert_close(xo.float().cpu().numpy(), xo_ref, f"X_out q={q}", tol)

        # backward on synthetic upstream gradient, with the oracle's own x_out / m as saved tensors
        xo32 = stored(xo_ref)
        m32 = stored(m_ref)
        d = dxo[p.local_gid]
        r1, r0, rdx, rdz = olayer.layer_backward(p, d, xo32, xl, m32, cols, h1, h0, o_act, True)
        dh1_ref += r1
        if sage:
            dh0_ref += r0
        dxl = torch.full((p.n_local, fi), float("nan"), dtype=tdt, device="cuda")
        dzh = torch.full((max(p.n_halo, 1), k), float("nan"), dtype=tdt, device="cuda")
        ctx.layer_bwd(layer, q, dev(d, tdt), dev(xo32, tdt), xld, z_dev if transform_first else dev(m32, tdt), h1d, h0d,
                      dh1_dev, dh0_dev, dxl, dzh if p.n_halo else None)
        assert_close(dxl.float().cpu().numpy(), rdx, f"dX_local q={q}", tol)
        if p.n_halo:
            assert_close(dzh.float().cpu().numpy(), rdz, f"dZ_halo q={q}", tol)
        halo_rows += p.n_halo
    # weight gradients: fp32 sums of products of stored values, no storage rounding on either side (transform first: the
    # transposed aggregate that enters the product is a stored bf16 tensor)
    assert_close(dh1_dev.cpu().numpy(), dh1_ref, "dH1 summed over partitions", tol if transform_first else TOL)
    if sage:
        assert_close(dh0_dev.cpu().numpy(), dh0_ref, "dH0 summed over partitions")
    st = ctx.stats()
    assert st["fwd_elems"][layer] == halo_rows * k and st["bwd_elems"][layer] == halo_rows * k
    assert st["full_fwd_elems"][layer] == halo_rows * fi
    ctx.close()


@pytest.mark.parametrize("conv", ["gcn", "sage"])
@pytest.mark.parametrize("fi,fo,ratio", [(16, 32, (4, 1)), (32, 8, (4, 1)), (128, 256, (1, 1)), (128, 256, (16, 1)),
                                         (256, 40, (8, 1)), (100, 256, (8, 1)), (256, 47, (8, 1)),
                                         (37, 19, (3, 1)), (512, 512, (32, 1)), (128, 64, (1569, 99))])
def test_layer_parity_small_graph(conv, fi, fo, ratio):
    g = synth.small_random_graph(1500, 9.0, conv, seed=fi + fo)
    part = synth.random_partition(g.n, 3, seed=5)
    _run_layer_case(g, part, 3, conv, fi, fo, ratio, vb.ACT_RELU, seed=fi * 3 + fo)


@pytest.mark.parametrize("conv,ratio", [("gcn", (1, 1)), ("gcn", (8, 1)), ("sage", (4, 1))])
def test_layer_parity_with_split_rows_and_identity_activation(conv, ratio):
    # hubs of degree ~1500 -> rows and transposed rows longer than one chunk, in local and halo parts
    g = hub_graph(6000, 4, 1500, 6.0, conv, seed=9)
    assert np.diff(g.rowptr).max() > 1000
    part = synth.random_partition(g.n, 2, seed=6)
    _run_layer_case(g, part, 2, conv, 64, 48, ratio, vb.ACT_IDENTITY, seed=77)


@pytest.mark.parametrize("conv", ["gcn", "sage"])
@pytest.mark.parametrize("fi,fo,ratio", [(100, 512, (1, 1)), (100, 512, (4, 1)), (100, 512, (32, 1)), (512, 512, (4, 1)),
                                         (512, 47, (32, 1)), (512, 47, (1, 1)), (37, 19, (3, 1)), (16, 32, (4, 1))])
def test_layer_parity_bf16_storage(conv, fi, fo, ratio):
    g = synth.small_random_graph(1500, 9.0, conv, seed=fi + fo)
    part = synth.random_partition(g.n, 3, seed=5)
    _run_layer_case(g, part, 3, conv, fi, fo, ratio, vb.ACT_RELU, seed=fi * 3 + fo, dtype="bf16")


@pytest.mark.parametrize("ratio", [(1, 1), (8, 1)])
def test_layer_parity_bf16_storage_with_split_rows(ratio):
    g = hub_graph(6000, 4, 1500, 6.0, "gcn", seed=9)
    part = synth.random_partition(g.n, 2, seed=6)
    _run_layer_case(g, part, 2, "gcn", 64, 48, ratio, vb.ACT_IDENTITY, seed=77, dtype="bf16")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("fi", [37, 101, 201, 511, 100, 512, 1024, 2048])
def test_layer_parity_with_few_local_entries_per_row(fi, dtype):
    """Eight random partitions keep about two entries per row local, so the transposed local block takes its
    short rows several to a wavefront, while the hubs' rows there still exceed one run and are split; the
    widths cover every number of loads per lane, with 4-element and with single-element accesses."""
    g = hub_graph(6000, 4, 1500, 6.0, "gcn", seed=12)
    part = synth.random_partition(g.n, 8, seed=3)
    host, _ = both_partitions(g, part, 8)
    assert all(hp.t_rowptr[hp.n_local] < 3 * hp.n_local for hp in host)
    assert max(int(np.diff(hp.t_rowptr[:hp.n_local + 1]).max()) for hp in host) > 64
    _run_layer_case(g, part, 8, "gcn", fi, 16, (4, 1), vb.ACT_RELU, seed=fi + 1, dtype=dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("fi,ratio", [(256, (2, 1)), (128, (1, 1))])
def test_layer_parity_with_compressed_rows_beyond_4_gib(fi, ratio, dtype):
    """The halo's rows lie more than 2^32 bytes into the compressed buffer (as with many millions of boundary
    rows): row offsets must be 64-bit there, for kept subsets and for whole rows."""
    k = omask.keep_count(fi, *ratio)
    shift = (1 << 32) // (k * (2 if dtype == "bf16" else 4)) + 1000
    g = synth.small_random_graph(1200, 8.0, "gcn", seed=31)
    part = synth.random_partition(g.n, 2, seed=2)
    _run_layer_case(g, part, 2, "gcn", fi, 64, ratio, vb.ACT_RELU, seed=fi, dtype=dtype, z_row_shift=shift)
    torch.cuda.empty_cache()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("fi,fo", [(2048, 64), (64, 2048)])
def test_layer_parity_at_the_maximum_width(fi, fo, dtype):
    g = synth.small_random_graph(700, 8.0, "sage", seed=fi // 64)
    part = synth.random_partition(g.n, 2, seed=3)
    _run_layer_case(g, part, 2, "sage", fi, fo, (8, 1), vb.ACT_RELU, seed=fi + 1, dtype=dtype)


@pytest.mark.parametrize("conv", ["gcn", "sage"])
def test_layer_parity_on_a_directed_operator(conv):
    # an operator with an arbitrary (non-symmetric) pattern and values: S and S^T must not be confused anywhere
    rng = np.random.default_rng(123)
    n = 1200
    pattern = rng.random((n, n)) < 0.006
    rowptr = np.concatenate(([0], np.cumsum(pattern.sum(axis=1)))).astype(np.int64)
    colidx = np.nonzero(pattern)[1].astype(np.int32)
    vals = rng.standard_normal(colidx.shape[0]).astype(np.float32)
    g = synth.Graph(n, rowptr, colidx, vals, 0, False)
    part = rng.integers(0, 3, size=n).astype(np.int32)              # uneven parts
    _run_layer_case(g, part, 3, conv, 96, 40, (4, 1), vb.ACT_RELU, seed=8)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_parity_after_a_partition_is_registered_again(dtype):
    """Registering a partition number a second time replaces everything derived from the first registration
    (launch plans, entry records, sizes): first a larger graph with long rows, then the one that is checked."""
    before = hub_graph(5000, 3, 900, 5.0, "sage", seed=21)
    host_before, _ = both_partitions(before, synth.random_partition(before.n, 3, seed=4), 3)
    g = synth.small_random_graph(1300, 7.0, "sage", seed=22)
    part = synth.random_partition(g.n, 3, seed=9)
    _run_layer_case(g, part, 3, "sage", 96, 40, (4, 1), vb.ACT_RELU, seed=5, dtype=dtype, registered_before=host_before)


@pytest.mark.parametrize("conv", ["gcn", "sage"])
@pytest.mark.parametrize("fi,fo,ratio", [(128, 47, (4, 1)), (512, 47, (1, 1)), (512, 33, (32, 1)), (64, 16, (3, 1)),
                                         (256, 64, (16, 1)), (16, 1, (2, 1))])
def test_layer_parity_in_the_transform_first_order(conv, fi, fo, ratio):
    # widths up to the limit of the halo kernels, outputs that are no multiple of anything, k a multiple of 8 (16-byte
    # chunks) and not (22 of 64: element by element), every element kept (dense copy), several tiles and a ragged last one
    g = synth.small_random_graph(1500, 9.0, conv, seed=fi + fo)
    part = synth.random_partition(g.n, 3, seed=fi)
    _run_layer_case(g, part, 3, conv, fi, fo, ratio, vb.ACT_IDENTITY, seed=fi * fo, dtype="bf16", transform_first=True)


def test_transform_first_edge_cases():
    # rows split over wavefronts in all three blocks; no halo at all; a partition that owns nothing and empty rows;
    # compressed rows far into the buffer (64-bit offsets)
    g = hub_graph(6000, 4, 1500, 6.0, "gcn", seed=9)
    _run_layer_case(g, synth.random_partition(g.n, 4, seed=10), 4, "gcn", 128, 47, (4, 1), vb.ACT_IDENTITY, seed=11,
                    dtype="bf16", transform_first=True)
    g = synth.small_random_graph(900, 8.0, "gcn", seed=2)
    _run_layer_case(g, np.zeros(g.n, dtype=np.int32), 1, "gcn", 64, 16, (4, 1), vb.ACT_IDENTITY, seed=3, dtype="bf16",
                    transform_first=True)
    g = synth.small_random_graph(400, 1.2, "sage", seed=4)
    part = synth.random_partition(g.n, 2, seed=1).astype(np.int32)
    part[part == 1] = 2
    _run_layer_case(g, part, 3, "sage", 32, 16, (2, 1), vb.ACT_IDENTITY, seed=5, dtype="bf16", transform_first=True)
    g = synth.small_random_graph(1200, 8.0, "gcn", seed=12)
    _run_layer_case(g, synth.random_partition(g.n, 3, seed=13), 3, "gcn", 512, 47, (1, 1), vb.ACT_IDENTITY, seed=14,
                    dtype="bf16", z_row_shift=(1 << 22) + 5, transform_first=True)


def test_layer_parity_single_partition_has_no_exchange():
    g = synth.small_random_graph(900, 8.0, "gcn", seed=2)
    part = np.zeros(g.n, dtype=np.int32)
    _run_layer_case(g, part, 1, "gcn", 64, 64, (4, 1), vb.ACT_RELU, seed=3)


def test_layer_parity_with_empty_partition_and_empty_rows():
    g = synth.small_random_graph(400, 1.2, "sage", seed=4)       # many isolated nodes -> empty rows
    part = synth.random_partition(g.n, 2, seed=1).astype(np.int32)
    part[part == 1] = 2                                           # partition 1 owns nothing
    _run_layer_case(g, part, 3, "sage", 32, 16, (2, 1), vb.ACT_RELU, seed=5)


def test_tiny_config_first_layer():
    w = synth.make_workload("tiny")
    _run_layer_case(w.graph, w.part, w.n_parts, "gcn", 16, 32, (4, 1), vb.ACT_RELU, seed=1, step=0, layer=1)


def test_forward_argument_errors_on_registered_partition():
    g = synth.small_random_graph(300, 6.0, "gcn", seed=8)
    part = synth.random_partition(g.n, 2, seed=1)
    host, _ = both_partitions(g, part, 2)
    ctx = vb.Context([16, 8], [vb.ACT_IDENTITY], vb.CONV_GCN, 2, KEY)
    ctx.register_partition(0, host[0])
    n = host[0].n_local
    x = torch.zeros((n, 16), device="cuda")
    h = torch.zeros((16, 8), device="cuda")
    o = torch.zeros((n, 8), device="cuda")
    m = torch.zeros((n, 16), device="cuda")
    z = torch.zeros((1, 16), device="cuda")
    for args in ((x, None, h, None, o, None, m),        # halo nodes but no compressed input
                 (x, z, h, h, o, None, m),              # h0 on a single-tap convolution
                 (x, z, None, None, o, None, m),        # no weights
                 (x, z, h, None, o, z, m)):             # z_out on the last layer
        with pytest.raises(vb.VarcoError) as e:
            ctx.layer_fwd(0, 0, *args)
        assert e.value.code == vb.ERR_INVALID_ARG
    with pytest.raises(vb.VarcoError) as e:
        ctx.layer_fwd(0, 1, x, z, h, None, o, None, m)  # partition 1 was never registered
    assert e.value.code == vb.ERR_STATE
    with pytest.raises(vb.VarcoError) as e:
        ctx.layer_bwd(0, 0, o, o, x, m, h, None, h, None, None, z)   # dz_halo without dx_local
    assert e.value.code == vb.ERR_INVALID_ARG
    # the compute calls allocate nothing: a stream without a prepared workspace set is a state error, on any call
    zin = torch.zeros((host[0].n_boundary + host[1].n_boundary, 16), device="cuda")
    side = torch.cuda.Stream()
    for call in (lambda st: ctx.layer_fwd(0, 0, x, zin, h, None, o, None, m, st),
                 lambda st: ctx.layer_bwd(0, 0, o, o, x, m, h, None, torch.zeros_like(h), None, None, None, st),
                 lambda st: ctx.aggregate_fwd(0, 0, x, zin, m, st),
                 lambda st: ctx.transform_fwd(0, x, h, o, False, False, st)):
        with pytest.raises(vb.VarcoError) as e:
            call(side)
        assert e.value.code == vb.ERR_STATE and "varco_prepare" in str(e.value)
    ctx.prepare(side)
    ctx.layer_fwd(0, 0, x, zin, h, None, o, None, m, side)
    side.synchronize()
    ctx.close()

    # rows wider than 512 elements: buffers that are not 16-byte aligned are refused before any launch
    wide = vb.Context([1024, 8], [vb.ACT_IDENTITY], vb.CONV_GCN, 2, KEY)
    wide.register_partition(0, host[0])
    flat = torch.zeros(n * 1024 + 4, device="cuda")
    xw, mw = flat[1:1 + n * 1024].view(n, 1024), torch.zeros((n, 1024), device="cuda")
    hw = torch.zeros((1024, 8), device="cuda")
    zw = torch.zeros((1, 1024), device="cuda")
    with pytest.raises(vb.VarcoError) as e:
        wide.layer_fwd(0, 0, xw, zw, hw, None, o, None, mw)
    assert e.value.code == vb.ERR_UNSUPPORTED
    wide.close()


def test_registration_rejects_malformed_index_arrays():
    """Nothing in a descriptor is trusted unchecked: unsorted or out-of-range columns, a transpose that does not
    hold the row block's entries, negative ids and a bad returned-row map are SHAPE errors at registration."""
    import copy
    g = synth.small_random_graph(400, 6.0, "gcn", seed=18)
    part = synth.random_partition(g.n, 2, seed=2)
    host, _ = both_partitions(g, part, 2)
    ctx = vb.Context([16, 8], [vb.ACT_IDENTITY], vb.CONV_GCN, 2, KEY)
    ctx.register_partition(0, host[0])                       # the well-formed partition is accepted
    good = host[1]
    row = int(np.argmax(np.diff(good.rowptr) >= 2))
    e0 = int(good.rowptr[row])

    def broken(change):
        hp = copy.copy(good)
        for name in ("colidx", "t_colidx", "t_vals", "halo_gid", "boundary_rows", "ret_src", "ret_ptr"):
            setattr(hp, name, getattr(good, name).copy())
        change(hp)
        return hp

    def swap_columns(hp):
        hp.colidx[e0], hp.colidx[e0 + 1] = hp.colidx[e0 + 1], hp.colidx[e0]

    def column_out_of_range(hp):
        hp.colidx[int(good.rowptr[row + 1]) - 1] = good.n_local + good.n_halo

    def transposed_row_out_of_range(hp):
        hp.t_colidx[0] = good.n_local

    def transposed_value_differs(hp):
        hp.t_vals[3] = np.float32(hp.t_vals[3] * 2 + 1)

    def negative_node_id(hp):
        hp.halo_gid[0] = -5

    def boundary_rows_descending(hp):
        hp.boundary_rows[:2] = hp.boundary_rows[:2][::-1]

    def negative_returned_row(hp):
        hp.ret_src[0] = -1

    def returned_pointer_too_short(hp):
        hp.ret_ptr[-1] -= 1

    for change, text in ((swap_columns, "ascending"), (column_out_of_range, "column outside"),
                         (transposed_row_out_of_range, "transposed entry outside"),
                         (transposed_value_differs, "differ from the row block"), (negative_node_id, "negative node id"),
                         (boundary_rows_descending, "boundary rows"), (negative_returned_row, "ret_src"),
                         (returned_pointer_too_short, "ret_ptr")):
        with pytest.raises(vb.VarcoError) as e:
            ctx.register_partition(1, broken(change))
        assert e.value.code == vb.ERR_SHAPE and text in str(e.value), (change.__name__, str(e.value))
    ctx.register_partition(1, good)
    ctx.close()
