"""GPU parity at the full size of the bf16-storage configuration (2,449,029 nodes, ~126.2 M directed entries
with self-loops, 32 random partitions, GCN 100 -> 512 -> 512 -> 47, ratios 1, 4 and 32). Inputs are bf16
values; the row-at-a-time oracle computes in fp64 and the device results (stored as bf16) are compared at the
bound of this configuration."""
import pytest
import torch

import large_common as lc

pytestmark = pytest.mark.gpu

BF16_TOL = 2.0 ** -7


@pytest.fixture(scope="module")
def large():
    d = lc.build_large("large_gcn_bf16")
    yield d
    d.clear()
    torch.cuda.empty_cache()


def test_partition_indexing_of_one_partition_is_bit_exact(large):
    lc.check_partition_indexing(large, 17)
    assert large["w"].ratios == ((1, 1), (4, 1), (32, 1))


@pytest.mark.parametrize("ratio", [(1, 1), (4, 1), (32, 1)])
@pytest.mark.parametrize("layer", [0, 1, 2])
def test_layer_forward_and_backward_on_sampled_rows(large, layer, ratio):
    lc.check_layer(large, layer, ratio, BF16_TOL, dh_cols=64, consumer=21)


@pytest.mark.parametrize("ratio", [(1, 1), (4, 1)])
def test_class_layer_with_the_transform_before_the_aggregation(large, ratio):
    # eq. (2) in the other order on the 512 -> 47 layer: the halo rows are transformed from their received elements
    # and rows of 47 elements are aggregated; same oracle rows, same counts
    lc.check_layer(large, 2, ratio, BF16_TOL, consumer=21, transform_first=True)
