"""A whole step captured in a HIP graph (step counter and key words on the device) replays bit for bit what the
same steps give when every call is issued eagerly."""
import numpy as np
import pytest
import torch

from gpu_common import KEY, both_partitions, hub_graph
from paper_2406_17611_amd import synth
from paper_2406_17611_amd.runner import PartitionedNetwork

pytestmark = pytest.mark.gpu


def _network(g, part, n_parts, widths, conv, n_streams, **kwargs):
    host, _ = both_partitions(g, part, n_parts)
    net = PartitionedNetwork(host, widths, conv, KEY, n_streams=n_streams, **kwargs)
    L = len(widths) - 1
    net.set_inputs(synth.features(g.n, widths[0], synth.SEED_FEAT))
    net.set_weights([synth.glorot(widths[l], widths[l + 1], synth.SEED_WEIGHT, 2 * l) for l in range(L)],
                    [synth.glorot(widths[l], widths[l + 1], synth.SEED_WEIGHT, 2 * l + 1) for l in range(L)])
    net.set_upstream(synth.upstream_grad(g.n, widths[-1], synth.SEED_GRAD))
    return net


def _snapshot(net):
    torch.cuda.synchronize()
    return [t.float().cpu().numpy().copy() for t in [net.x[-1], net.dx[1]] + net.dh1 + [h for h in net.dh0 if h is not None]]


@pytest.mark.parametrize("n_streams", [1, 2])
def test_graph_replays_equal_eager_steps(n_streams):
    g = hub_graph(5000, 3, 1200, 7.0, "sage", seed=15)       # includes rows split over wavefronts (fix-up launches)
    part = synth.random_partition(g.n, 4, seed=16)
    widths, ratio, first = (64, 128, 128, 16), (4, 1), 100
    eager = _network(g, part, 4, widths, "sage", n_streams)
    want = []
    for t in range(first + 1, first + 4):
        eager.zero_grads()
        eager.step(t, ratio)
        want.append(_snapshot(eager))

    net = _network(g, part, 4, widths, "sage", n_streams)
    graph = net.capture_step(ratio)
    net.ctx.set_step(first)                                   # the first replay advances to first + 1
    scratch = torch.zeros(1 << 20, device="cuda")
    for i in range(3):
        net.zero_grads()                                      # eager work between the replays
        scratch.add_(1.0)
        torch.cuda.synchronize()
        graph.replay()
        got = _snapshot(net)
        for a, b in zip(got, want[i]):
            assert np.array_equal(a, b), f"replay {i}"
    assert float(scratch[0].item()) == 3.0
    # eager calls keep working after the capture, on the device-resident step
    net.zero_grads()
    net.step(first + 1, ratio)
    for a, b in zip(_snapshot(net), want[0]):
        assert np.array_equal(a, b)


def test_graph_replays_with_the_class_layer_transforming_first():
    # bf16 storage, the last layer in the order S (X H): its halo kernels read the step's key words from the device
    # table like every other hashing kernel, so replays follow the steps
    g = hub_graph(5000, 3, 1200, 7.0, "gcn", seed=25)
    part = synth.random_partition(g.n, 4, seed=26)
    widths, ratio, first = (64, 128, 128, 16), (4, 1), 40
    kw = dict(dtype="bf16", transform_first=(2,))
    eager = _network(g, part, 4, widths, "gcn", 1, **kw)
    want = []
    for t in range(first + 1, first + 4):
        eager.zero_grads()
        eager.step(t, ratio)
        want.append(_snapshot(eager))
    assert not np.array_equal(want[0][1], want[1][1])         # the kept positions change from step to step
    net = _network(g, part, 4, widths, "gcn", 1, **kw)
    graph = net.capture_step(ratio)
    net.ctx.set_step(first)
    for i in range(3):
        net.zero_grads()
        torch.cuda.synchronize()
        graph.replay()
        for a, b in zip(_snapshot(net), want[i]):
            assert np.array_equal(a, b), f"replay {i}"
