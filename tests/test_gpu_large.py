"""GPU parity at the full size of the large fp32 configuration (2,449,029 nodes, ~123.7 M directed entries,
8 random partitions, SAGE-mean 100 -> 256 -> 256 -> 47, ratio 8)."""
import pytest
import torch

import large_common as lc
from gpu_common import TOL

pytestmark = pytest.mark.gpu

RATIO = (8, 1)


@pytest.fixture(scope="module")
def large():
    d = lc.build_large("large_sage")
    yield d
    d.clear()
    torch.cuda.empty_cache()


def test_partition_indexing_of_one_partition_is_bit_exact(large):
    lc.check_partition_indexing(large, 3)
    # Table 1's law for equal random parts: share of entries inside a partition = (2E/P) / 2E here (no self-loops)
    w, g, host = large["w"], large["g"], large["host"]
    inside = sum(int((h.colidx < h.n_local).sum()) for h in host) / g.nnz
    assert abs(inside - 1.0 / w.n_parts) < 2e-3


@pytest.mark.parametrize("layer", [0, 1, 2])
def test_layer_forward_and_backward_on_sampled_rows(large, layer):
    lc.check_layer(large, layer, RATIO, TOL)
