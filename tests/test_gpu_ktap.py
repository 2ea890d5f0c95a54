"""GPU parity of general K-tap layers (one compressed exchange per hop) built from the library's
building-block calls, against the K-tap oracle."""
import numpy as np
import pytest
import torch

from gpu_common import KEY, TOL, assert_close, both_partitions
from oracle import ktap as oktap
from oracle import layer as olayer
from oracle import mask as omask
from oracle.rounding import round_bf16
from paper_2406_17611_amd import synth
from paper_2406_17611_amd.runner import KTapNetwork

pytestmark = pytest.mark.gpu


def _gather(parts, per_part, n):
    out = np.empty((n, per_part[0].shape[1]))
    for p in parts:
        out[p.local_gid] = per_part[p.q]
    return out


@pytest.mark.parametrize("n_taps,ratio,dtype", [(3, (4, 1), "f32"), (4, (2, 1), "f32"), (3, (1, 1), "f32"), (2, (8, 1), "f32"),
                                                (1, (4, 1), "f32"), (3, (1, 0), "f32"), (3, (4, 1), "bf16")])
def test_ktap_network(n_taps, ratio, dtype):
    g = synth.small_random_graph(2500, 9.0, "sage", seed=70 + n_taps)
    part = synth.random_partition(g.n, 3, seed=71)
    host, orc = both_partitions(g, part, 3)
    widths = (64, 128, 24)
    L = 2
    bf16 = dtype == "bf16"
    # bf16: the sum of K products is rounded after every product, each hop's aggregate once more
    tol = 2.0 ** -6 if bf16 else TOL
    x0 = synth.features(g.n, widths[0], synth.SEED_FEAT)
    dxl = synth.upstream_grad(g.n, widths[-1], synth.SEED_GRAD)
    if bf16:
        x0, dxl = round_bf16(x0).astype(np.float32), round_bf16(dxl).astype(np.float32)
    weights = [[synth.glorot(widths[l], widths[l + 1], synth.SEED_WEIGHT, 8 * l + hop) for hop in range(n_taps)]
               for l in range(L)]
    net = KTapNetwork(host, widths, n_taps, KEY, dtype=dtype)
    net.set_inputs(x0)
    net.set_tap_weights(weights)
    net.set_upstream(dxl)
    acts = [olayer.RELU, olayer.IDENTITY]
    keep = [omask.keep_count(w, *ratio) for w in widths[:-1]]
    step = 5
    ref = oktap.network_step(orc, [x0[p.local_gid] for p in orc], weights, acts, keep, KEY, step,
                             [dxl[p.local_gid] for p in orc])
    net.zero_grads()
    net.ctx.reset_stats()
    net.forward(step, ratio)
    torch.cuda.synchronize()
    for l in range(L):
        for hop in range(1, n_taps):
            assert_close(net.to_global(net.y[l][hop]), _gather(orc, ref["y"][l][hop], g.n), f"Y_{l},{hop}", tol)
        assert_close(net.to_global(net.x[l + 1]), _gather(orc, ref["x"][l + 1], g.n), f"X_{l + 1}", tol)
    # the ReLU gates of the backward pass are taken on the oracle's stored activations (as in the network tests)
    stored = (lambda a: round_bf16(a).astype(np.float32)) if bf16 else (lambda a: np.asarray(a, dtype=np.float32))
    for l in range(L):
        net.x[l + 1].copy_(torch.from_numpy(stored(np.vstack(ref["x"][l + 1]))))
        for hop in range(1, n_taps):
            net.y[l][hop].copy_(torch.from_numpy(stored(np.vstack(ref["y"][l][hop]))))
    net.backward()
    torch.cuda.synchronize()
    for l in range(L):
        for hop in range(n_taps):
            assert_close(net.dh[l][hop].cpu().numpy(), ref["dh"][l][hop], f"dH_{l},{hop}", tol)
    assert_close(net.to_global(net.dx[1]), _gather(orc, ref["dx"][1], g.n), "dX_1", tol)
    st = net.ctx.stats()
    assert st["fwd_elems"] == ref["fwd_elems"] and st["bwd_elems"] == ref["bwd_elems"]
