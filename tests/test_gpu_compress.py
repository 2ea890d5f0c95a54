"""GPU parity of the encoder / decoder (Definition 1, Appendix A): pure copies, compared bit for bit."""
import numpy as np
import pytest
import torch

from gpu_common import KEY, dev
from oracle import layer as olayer
from oracle import mask as omask
from oracle.rounding import round_bf16
from paper_2406_17611_amd import binding as vb

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("width,ratio", [(16, (4, 1)), (32, (4, 1)), (100, (8, 1)), (100, (32, 1)), (128, (16, 1)),
                                          (128, (1569, 99)), (256, (8, 1)), (256, (1, 1)), (512, (32, 1)),
                                          (512, (4, 1)), (7, (2, 1)), (1, (1, 1)), (100, (128, 1)), (2048, (3, 1)),
                                          (37, (3, 2))])
def test_compress_decompress_bit_exact(width, ratio):
    rng = np.random.default_rng(width * 7 + ratio[0])
    n_src, n_rows, ldx = 5000, 3001, width + 3
    x = rng.standard_normal((n_src, ldx)).astype(np.float32)
    rows = rng.permutation(n_src)[:n_rows].astype(np.int32)
    gids = rng.integers(0, 2_449_029, size=n_rows).astype(np.int32)
    step, layer = 12, 1
    ctx = vb.Context([8, width, 8], [1, 0], vb.CONV_GCN, 1, KEY)
    ctx.prepare()
    ctx.begin_step(step)
    ctx.set_ratio(layer, *ratio)
    k = ctx.keep(layer)
    assert k == omask.keep_count(width, *ratio)
    cols = omask.kept_columns(gids, width, k, KEY, step, layer)

    xd, rd, gd = dev(x), dev(rows), dev(gids)
    z = torch.full((n_rows, k), float("nan"), dtype=torch.float32, device="cuda")
    ctx.compress(layer, gd, rd, n_rows, xd, ldx, z)
    want_z = olayer.compress(x, rows, cols).astype(np.float32)
    assert np.array_equal(z.cpu().numpy(), want_z)

    # rows = NULL means row i
    z2 = torch.empty((n_rows, k), dtype=torch.float32, device="cuda")
    ctx.compress(layer, gd, None, n_rows, xd, ldx, z2)
    assert np.array_equal(z2.cpu().numpy(), olayer.compress(x, np.arange(n_rows), cols).astype(np.float32))

    # decoder: kept values in place, zero elsewhere, untouched padding columns and other rows
    out = torch.full((n_src, ldx), 7.0, dtype=torch.float32, device="cuda")
    ctx.decompress(layer, gd, rd, n_rows, z, out, ldx, 0)
    want = np.full((n_src, ldx), 7.0, dtype=np.float32)
    want[rows, :width] = olayer.decompress(want_z.astype(np.float64), cols, width).astype(np.float32)
    assert np.array_equal(out.cpu().numpy(), want)

    # owner-side accumulation of returned values (single fp32 add per element: exact match expected)
    acc = dev(x.copy())
    ctx.decompress(layer, gd, rd, n_rows, z, acc, ldx, 1)
    want_acc = x.copy()
    for i in range(n_rows):
        want_acc[rows[i], cols[i]] += want_z[i]
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    ctx.close()


@pytest.mark.parametrize("width,ratio", [(16, (4, 1)), (100, (4, 1)), (512, (4, 1)), (512, (32, 1)), (512, (1, 1)),
                                          (37, (3, 2)), (2048, (3, 1))])
def test_compress_decompress_bit_exact_bf16_storage(width, ratio):
    """bf16 storage: the encoder and decoder copy 2-byte elements; the owner-side add is one fp32 add of two bf16
    values rounded to bf16 once, which the oracle's rounding reproduces exactly."""
    rng = np.random.default_rng(width * 11 + ratio[0])
    n_src, n_rows, ldx = 4000, 2501, width + 2
    x = round_bf16(rng.standard_normal((n_src, ldx))).astype(np.float32)
    rows = rng.permutation(n_src)[:n_rows].astype(np.int32)
    gids = rng.integers(0, 2_449_029, size=n_rows).astype(np.int32)
    step, layer = 9, 1
    ctx = vb.Context([8, width, 8], [1, 0], vb.CONV_GCN, 1, KEY, vb.BF16)
    ctx.prepare()
    ctx.begin_step(step)
    ctx.set_ratio(layer, *ratio)
    k = ctx.keep(layer)
    cols = omask.kept_columns(gids, width, k, KEY, step, layer)
    bf = torch.bfloat16
    xd, rd, gd = dev(x, bf), dev(rows), dev(gids)
    z = torch.full((n_rows, k), float("nan"), dtype=bf, device="cuda")
    ctx.compress(layer, gd, rd, n_rows, xd, ldx, z)
    want_z = olayer.compress(x, rows, cols).astype(np.float32)
    assert np.array_equal(z.float().cpu().numpy(), want_z)
    out = torch.full((n_src, ldx), 7.0, dtype=bf, device="cuda")
    ctx.decompress(layer, gd, rd, n_rows, z, out, ldx, 0)
    want = np.full((n_src, ldx), 7.0, dtype=np.float32)
    want[rows, :width] = olayer.decompress(want_z.astype(np.float64), cols, width).astype(np.float32)
    assert np.array_equal(out.float().cpu().numpy(), want)
    acc = dev(x.copy(), bf)
    ctx.decompress(layer, gd, rd, n_rows, z, acc, ldx, 1)
    want_acc = x.astype(np.float64)
    for i in range(n_rows):
        want_acc[rows[i], cols[i]] += want_z[i]
    assert np.array_equal(acc.float().cpu().numpy(), round_bf16(want_acc).astype(np.float32))
    ctx.close()


def test_unbounded_ratio_sends_nothing_and_decodes_to_zero():
    ctx = vb.Context([8, 64, 8], [1, 0], vb.CONV_GCN, 1, KEY)
    ctx.prepare()
    ctx.begin_step(0)
    ctx.set_ratio(1, 1, 0)
    assert ctx.keep(1) == 0
    rows = dev(np.array([3, 0, 7], dtype=np.int32))
    gids = dev(np.array([11, 12, 13], dtype=np.int32))
    x = torch.full((9, 64), 5.0, device="cuda")
    ctx.compress(1, gids, rows, 3, x, 64, None)          # nothing to write: the buffer may be NULL
    ctx.decompress(1, gids, rows, 3, None, x, 64, 0)     # decoder: the listed rows become zero
    want = np.full((9, 64), 5.0, dtype=np.float32)
    want[[3, 0, 7]] = 0.0
    assert np.array_equal(x.cpu().numpy(), want)
    ctx.decompress(1, gids, rows, 3, None, x, 64, 1)     # nothing returned, nothing added
    assert np.array_equal(x.cpu().numpy(), want)
    ctx.close()


def test_mask_changes_with_step_and_layer_like_the_oracle():
    width, k_ratio = 128, (8, 1)
    rng = np.random.default_rng(0)
    n = 2000
    x = rng.standard_normal((n, width)).astype(np.float32)
    gids = np.arange(n, dtype=np.int32) * 1223
    ctx = vb.Context([width, width, 8], [1, 0], vb.CONV_GCN, 1, KEY ^ 0x55)
    ctx.prepare()
    xd, gd = dev(x), dev(gids)
    for step in (0, 1, 2 ** 40 + 5):
        for layer in (0, 1):
            ctx.begin_step(step)
            ctx.set_ratio(-1, *k_ratio)
            k = ctx.keep(layer)
            z = torch.empty((n, k), dtype=torch.float32, device="cuda")
            ctx.compress(layer, gd, None, n, xd, width, z)
            cols = omask.kept_columns(gids, width, k, KEY ^ 0x55, step, layer)
            assert np.array_equal(z.cpu().numpy(), x[np.arange(n)[:, None], cols])
    ctx.close()


def test_ratio_change_inside_a_step_is_refused():
    ctx = vb.Context([16, 8], [0], vb.CONV_GCN, 1, KEY)
    ctx.prepare()
    ctx.begin_step(0)
    ctx.set_ratio(0, 4, 1)
    x = torch.zeros((4, 16), device="cuda")
    g = torch.arange(4, dtype=torch.int32, device="cuda")
    z = torch.empty((4, 4), device="cuda")
    ctx.compress(0, g, None, 4, x, 16, z)
    with pytest.raises(vb.VarcoError) as e:
        ctx.set_ratio(0, 2, 1)
    assert e.value.code == vb.ERR_STATE
    ctx.begin_step(1)
    ctx.set_ratio(0, 2, 1)
    with pytest.raises(vb.VarcoError) as e:
        ctx.compress(0, g, None, 4, x, 8, z)                  # ldx below the width
    assert e.value.code == vb.ERR_SHAPE
    ctx.close()
