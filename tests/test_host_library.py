"""CPU-only checks of the HIP library's host side: it loads, exports what include/varco.h declares, its
partition builder is bit-identical to the oracle's, and host-checkable errors come back as status codes."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import mask as omask
from oracle import partition as opart
from paper_2406_17611_amd import binding as vb
from paper_2406_17611_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "varco.h")).read()
    declared = set(re.findall(r"\b(varco_[a-z_]+)\s*\(", header))
    assert declared == set(vb.EXPORTS)
    L = C.CDLL(vb.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


_ARRAYS = ["rowptr", "colidx", "vals", "t_rowptr", "t_colidx", "t_vals", "local_gid", "halo_gid", "halo_owner_ptr",
           "boundary_rows", "halo_src_row", "halo_zrow"]


def _assert_same(host_parts, oracle_parts):
    assert len(host_parts) == len(oracle_parts)
    for hp, op in zip(host_parts, oracle_parts):
        assert (hp.n_local, hp.n_halo, hp.n_boundary, hp.z_row_offset, hp.nnz) == \
               (op.n_local, op.n_halo, op.n_boundary, op.z_row_offset, op.nnz)
        for name in _ARRAYS:
            a, b = getattr(hp, name), getattr(op, name)
            assert a.dtype == b.dtype, name
            assert np.array_equal(a, b), name                      # bit-exact, values included
        assert hp.halo_row_offset == op.halo_row_offset
    # the owners' reverse map of the backward exchange
    for hp, (ptr, src) in zip(host_parts, opart.returned_row_map(oracle_parts)):
        assert hp.n_returned == src.shape[0]
        for a, b in ((hp.ret_ptr, ptr), (hp.ret_src, src)):
            assert a.dtype == b.dtype and np.array_equal(a, b)


@pytest.mark.parametrize("conv", ["gcn", "sage"])
@pytest.mark.parametrize("n_parts", [1, 2, 5, 16])
def test_partition_builder_matches_oracle_small(conv, n_parts):
    g = synth.small_random_graph(700, 7.0, conv, seed=11)
    part = synth.random_partition(g.n, n_parts, seed=12)
    hp = vb.partition_build(g.n, g.rowptr, g.colidx, g.vals, part, n_parts)
    op = opart.build_partitions(g.n, g.rowptr, g.colidx, g.vals, part, n_parts)
    _assert_same(hp, op)


def test_partition_builder_handles_empty_partition_and_isolated_nodes():
    g = synth.small_random_graph(50, 1.0, "sage", seed=3)          # sparse: some empty rows
    part = np.zeros(g.n, dtype=np.int32)
    part[25:] = 2                                                   # partition 1 owns nothing
    hp = vb.partition_build(g.n, g.rowptr, g.colidx, g.vals, part, 3)
    op = opart.build_partitions(g.n, g.rowptr, g.colidx, g.vals, part, 3)
    _assert_same(hp, op)
    assert hp[1].n_local == 0 and hp[1].nnz == 0


def test_partition_builder_matches_oracle_on_random_directed_graphs():
    """Random small operators that need not be symmetric (the builder and the oracle must agree on any sparsity
    pattern with ascending columns): uneven and empty partitions, isolated nodes, self-loops, dense rows."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=60, deadline=None)
    @given(st.integers(1, 40), st.integers(1, 6), st.floats(0.0, 0.6), st.integers(0, 2**31 - 1))
    def check(n, n_parts, density, seed):
        rng = np.random.default_rng(seed)
        pattern = rng.random((n, n)) < density
        rowptr = np.concatenate(([0], np.cumsum(pattern.sum(axis=1)))).astype(np.int64)
        colidx = np.nonzero(pattern)[1].astype(np.int32)               # ascending within a row
        vals = rng.standard_normal(colidx.shape[0]).astype(np.float32)
        part = rng.integers(0, n_parts, size=n).astype(np.int32)       # any map: uneven, possibly empty parts
        hp = vb.partition_build(n, rowptr, colidx, vals, part, n_parts)
        op = opart.build_partitions(n, rowptr, colidx, vals, part, n_parts)
        _assert_same(hp, op)

    check()


@pytest.mark.parametrize("name", ["tiny", "medium", "medium_bfs16"])
def test_partition_builder_matches_oracle_on_configs(name):
    w = synth.make_workload(name)
    g = w.graph
    hp = vb.partition_build(g.n, g.rowptr, g.colidx, g.vals, w.part, w.n_parts)
    op = opart.build_partitions(g.n, g.rowptr, g.colidx, g.vals, w.part, w.n_parts)
    _assert_same(hp, op)


def test_partition_builder_rejects_bad_input():
    g = synth.small_random_graph(40, 4.0, "gcn", seed=1)
    part = synth.random_partition(g.n, 2, 2)
    bad = part.copy()
    bad[3] = 2
    with pytest.raises(vb.VarcoError) as e:
        vb.partition_build(g.n, g.rowptr, g.colidx, g.vals, bad, 2)
    assert e.value.code == vb.ERR_INVALID_ARG
    cols = g.colidx.copy()
    r = int(np.argmax(np.diff(g.rowptr) >= 2))
    cols[g.rowptr[r]], cols[g.rowptr[r] + 1] = cols[g.rowptr[r] + 1], cols[g.rowptr[r]]
    with pytest.raises(vb.VarcoError) as e:
        vb.partition_build(g.n, g.rowptr, cols, g.vals, part, 2)
    assert e.value.code == vb.ERR_INVALID_ARG and "ascending" in str(e.value)
    cols = g.colidx.copy()
    cols[0] = g.n
    with pytest.raises(vb.VarcoError):
        vb.partition_build(g.n, g.rowptr, cols, g.vals, part, 2)


def test_create_argument_errors():
    def make(widths, act, conv=vb.CONV_GCN, parts=2, dtype=vb.F32):
        return vb.Context(widths, act, conv, parts, 1, dtype)
    with pytest.raises(vb.VarcoError) as e:
        make([16, 0], [1])
    assert e.value.code == vb.ERR_SHAPE
    with pytest.raises(vb.VarcoError) as e:
        make([16, 8], [7])
    assert e.value.code == vb.ERR_UNSUPPORTED
    with pytest.raises(vb.VarcoError) as e:
        make([16, 8], [1], conv=5)
    assert e.value.code == vb.ERR_UNSUPPORTED
    with pytest.raises(vb.VarcoError) as e:
        make([16, 8], [1], dtype=3)
    assert e.value.code == vb.ERR_UNSUPPORTED
    with pytest.raises(vb.VarcoError) as e:
        make([16, 8], [1], parts=0)
    assert e.value.code == vb.ERR_INVALID_ARG
    with pytest.raises(vb.VarcoError) as e:
        make([1022, 8], [1])                                          # wide and not a multiple of 4
    assert e.value.code == vb.ERR_UNSUPPORTED
    with pytest.raises(vb.VarcoError) as e:
        make([4, 4] * 9, [1] * 17)
    assert e.value.code == vb.ERR_INVALID_ARG


def test_ratio_to_keep_count_matches_oracle_and_rejects_expansion():
    widths = [100, 256, 128, 47]
    ctx = vb.Context(widths, [1, 1, 0], vb.CONV_SAGE, 4, 99)
    assert [ctx.keep(l) for l in range(3)] == widths[:3]             # created at ratio 1
    for num, den in ((1, 1), (2, 1), (8, 1), (32, 1), (128, 1), (1000, 1), (3, 2), (1584 - 15 * 41, 99), (114, 99)):
        ctx.set_ratio(-1, num, den)
        for l in range(3):
            assert ctx.keep(l) == omask.keep_count(widths[l], num, den)
    ctx.set_ratio(1, 4, 1)
    assert ctx.keep(1) == 64 and ctx.keep(0) == omask.keep_count(100, 114, 99)
    for num, den in ((1, 2), (0, 1), (0, 0)):
        with pytest.raises(vb.VarcoError) as e:
            ctx.set_ratio(-1, num, den)
        assert e.value.code == vb.ERR_INVALID_ARG
    ctx.set_ratio(2, 1, 0)                                           # unbounded ratio: no communication
    assert ctx.keep(2) == 0 == omask.keep_count(128, 1, 0) and ctx.keep(1) == 64
    with pytest.raises(vb.VarcoError) as e:
        ctx.set_ratio(3, 2, 1)
    assert e.value.code == vb.ERR_INVALID_ARG
    with pytest.raises(vb.VarcoError) as e:
        ctx.keep(-1)
    assert e.value.code == vb.ERR_INVALID_ARG
    ctx.close()


def test_calls_on_unregistered_partition_are_state_errors():
    ctx = vb.Context([8, 4], [0], vb.CONV_GCN, 2, 1)
    L = vb.lib()
    rc = L.varco_layer_fwd(ctx._h, 0, 1, None, None, None, None, None, None, None, None)
    assert rc == vb.ERR_STATE
    rc = L.varco_layer_fwd(ctx._h, 0, 2, None, None, None, None, None, None, None, None)
    assert rc == vb.ERR_INVALID_ARG
    rc = L.varco_layer_bwd(ctx._h, 1, 0, *([None] * 11))
    assert rc == vb.ERR_INVALID_ARG and b"layer" in L.varco_last_error(ctx._h)
    rc = L.varco_compress(ctx._h, 0, None, None, 5, None, 8, None, None)
    assert rc == vb.ERR_INVALID_ARG
    rc = L.varco_compress(ctx._h, 0, None, None, -1, None, 8, None, None)
    assert rc == vb.ERR_SHAPE
    rc = L.varco_decompress(ctx._h, 0, None, None, 0, None, None, 8, 2, None)
    assert rc == vb.ERR_INVALID_ARG
    assert L.varco_compress(ctx._h, 0, None, None, 0, None, 8, None, None) == vb.OK     # empty input is a no-op
    assert L.varco_begin_step(None, 0) == vb.ERR_INVALID_ARG
    ctx.close()


def test_compute_calls_never_allocate_and_fail_without_a_prepared_stream():
    """The compute calls take their device state from varco_prepare / varco_register_partition; on a context that
    never saw either they return a state error before touching any device (so this runs without a GPU)."""
    ctx = vb.Context([8, 4, 3], [1, 0], vb.CONV_SAGE, 2, 1)
    L = vb.lib()
    a = np.zeros(64, dtype=np.float32)
    p = a.ctypes.data
    for rc in (L.varco_compress(ctx._h, 0, p, None, 2, p, 8, p, None),
               L.varco_decompress(ctx._h, 0, p, None, 2, p, p, 8, 0, None),
               L.varco_transform_fwd(ctx._h, 0, 2, p, p, p, 0, 0, None),
               L.varco_transform_bwd_weight(ctx._h, 0, 2, p, p, p, p, None),
               L.varco_transform_bwd_input(ctx._h, 0, 2, p, p, p, p, 0, None)):
        assert rc == vb.ERR_STATE
        assert b"varco_prepare" in L.varco_last_error(ctx._h)
    assert L.varco_prepare(None, None) == vb.ERR_INVALID_ARG
    # changing the ratio on a context without workspace sets stays a pure host call
    ctx.set_ratio(-1, 4, 1)
    assert ctx.keep(0) == 2
    ctx.close()


def test_schedules_match_the_oracle_exactly():
    for step in range(0, 301, 7):
        assert vb.schedule_ratio(vb.SCHED_LINEAR, step, 300, 128, 1, 5) == omask.linear_ratio(128, 1, 5, 300, step)
        assert vb.schedule_ratio(vb.SCHED_LINEAR, step, 300, 16, 2, 1) == omask.linear_ratio(16, 2, 1, 300, step)
        assert vb.schedule_ratio(vb.SCHED_FIXED_INCREMENT, step, 300, 64, 1, 1) == omask.fixed_increment_ratio(64, -1, 1, step)
        assert vb.schedule_ratio(vb.SCHED_EXPONENTIAL, step, 300, 128, 1, 2) == omask.exponential_ratio(2, 128, 1, 300, step)
    for step in range(0, 11):
        assert vb.schedule_ratio(vb.SCHED_EXPONENTIAL, step, 10, 100, 5, 3) == omask.exponential_ratio(3, 100, 5, 10, step)
    num, den = vb.schedule_ratio(vb.SCHED_LINEAR, 50, 99, 16, 1, 1)                       # the 16-partition configuration:
    assert num * 99 == (1584 - 15 * 50) * den and (num, den) == (278, 33)                 # (1584 - 15 t) / 99 in lowest terms
    for args in ((vb.SCHED_LINEAR, 0, 0, 8, 1, 1), (vb.SCHED_LINEAR, -1, 10, 8, 1, 1), (vb.SCHED_LINEAR, 0, 10, 1, 2, 1),
                 (vb.SCHED_LINEAR, 0, 10, 8, 0, 1), (vb.SCHED_EXPONENTIAL, 0, 10, 8, 1, 1), (7, 0, 10, 8, 1, 1)):
        with pytest.raises(vb.VarcoError) as e:
            vb.schedule_ratio(*args)
        assert e.value.code == vb.ERR_INVALID_ARG


def test_layer_order_is_accepted_only_where_the_kernels_cover_it():
    L = vb.lib()
    ctx = vb.Context([100, 512, 47], [1, 0], vb.CONV_GCN, 2, 1, vb.BF16)
    assert L.varco_set_layer_order(ctx._h, 1, vb.ORDER_TRANSFORM_FIRST) == vb.OK
    assert L.varco_set_layer_order(ctx._h, 1, vb.ORDER_AGGREGATE_FIRST) == vb.OK
    assert L.varco_set_layer_order(ctx._h, 1, 2) == vb.ERR_INVALID_ARG
    assert L.varco_set_layer_order(ctx._h, 2, vb.ORDER_TRANSFORM_FIRST) == vb.ERR_INVALID_ARG      # no such layer
    assert L.varco_set_layer_order(ctx._h, 0, vb.ORDER_TRANSFORM_FIRST) == vb.ERR_UNSUPPORTED      # ReLU layer, 512 outputs
    assert L.varco_set_layer_order(None, 0, 0) == vb.ERR_INVALID_ARG
    ctx.close()
    ctx = vb.Context([100, 512, 47], [1, 0], vb.CONV_GCN, 2, 1, vb.F32)
    assert L.varco_set_layer_order(ctx._h, 1, vb.ORDER_TRANSFORM_FIRST) == vb.ERR_UNSUPPORTED      # fp32 storage
    assert b"bf16" in vb.lib().varco_last_error(ctx._h)
    ctx.close()
    ctx = vb.Context([100, 510, 47], [1, 0], vb.CONV_SAGE, 2, 1, vb.BF16)
    assert L.varco_set_layer_order(ctx._h, 1, vb.ORDER_TRANSFORM_FIRST) == vb.ERR_UNSUPPORTED      # width not a multiple of 4
    ctx.close()


def test_host_checkable_errors_of_the_building_block_and_training_calls():
    ctx = vb.Context([8, 4, 3], [1, 0], vb.CONV_SAGE, 2, 1)
    L = vb.lib()
    h = ctx._h
    assert L.varco_aggregate_fwd(h, vb.tap(0, 1), 1, None, None, None, None) == vb.ERR_STATE        # not registered
    assert L.varco_aggregate_fwd(h, vb.tap(2, 1), 0, None, None, None, None) == vb.ERR_INVALID_ARG  # no such layer
    assert L.varco_aggregate_bwd(h, -1, 0, None, None, None, None) == vb.ERR_INVALID_ARG
    assert L.varco_aggregate_bwd(h, 16 * 16, 0, None, None, None, None) == vb.ERR_INVALID_ARG       # hop out of range
    assert L.varco_compress(h, vb.tap(1, 3), None, None, 0, None, 8, None, None) == vb.OK            # hop addresses are accepted
    assert L.varco_transform_fwd(h, 2, 10, None, None, None, 0, 0, None) == vb.ERR_INVALID_ARG      # layer
    assert L.varco_transform_fwd(h, 0, -1, None, None, None, 0, 0, None) == vb.ERR_SHAPE
    assert L.varco_transform_fwd(h, 0, 10, None, None, None, 0, 0, None) == vb.ERR_INVALID_ARG      # null pointers
    assert L.varco_transform_fwd(h, 0, 0, None, None, None, 0, 0, None) == vb.OK                    # no rows: no-op
    assert L.varco_transform_bwd_weight(h, 0, 10, None, None, None, None, None) == vb.ERR_INVALID_ARG
    assert L.varco_transform_bwd_input(h, 1, 10, None, None, None, None, 0, None) == vb.ERR_INVALID_ARG
    assert L.varco_softmax_xent(h, None, 3, None, 10, 3, 1.0, None, 3, None, None, None, None) == vb.ERR_INVALID_ARG
    assert L.varco_softmax_xent(h, None, 2, None, 10, 3, 1.0, None, 3, None, None, None, None) == vb.ERR_SHAPE   # ld < classes
    assert L.varco_softmax_xent(h, None, 3, None, -1, 3, 1.0, None, 3, None, None, None, None) == vb.ERR_SHAPE
    assert L.varco_softmax_xent(h, None, 3, None, 0, 3, 1.0, None, 3, None, None, None, None) == vb.OK
    assert L.varco_softmax_xent(None, None, 3, None, 0, 3, 1.0, None, 3, None, None, None, None) == vb.ERR_INVALID_ARG
    assert L.varco_sgd_step(None, None, 5, 0.1, None) == vb.ERR_INVALID_ARG
    assert L.varco_sgd_step(None, None, -5, 0.1, None) == vb.ERR_SHAPE
    assert L.varco_sgd_step(None, None, 0, 0.1, None) == vb.OK
    assert L.varco_sum_gradients(None, None, 5, None) == vb.ERR_INVALID_ARG
    ctx.close()
