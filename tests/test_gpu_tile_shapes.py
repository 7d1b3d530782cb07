"""Every block shape of the bf16 transfer kernel (tile, wave grid, k groups) on the same small layers, forced
through the test aid of include/flop_bench.h: ragged tile and k tails, k extents shorter than one round of the
groups, odd extents inside 16-byte rows, the fused column sums, and the riding entry points (block sizes up to
1024 threads carry the 256-thread boundary blocks)."""
import numpy as np
import pytest
import torch

from paper_1910_04732_amd import flop, synth
from test_gpu_parity import check_layer
from test_gpu_riders import CASES, test_training_step_through_riders as rider_step

pytestmark = pytest.mark.gpu


@pytest.fixture
def forced_shape(request):
    flop.flop_bench_force_tile_shape(request.param)
    yield request.param
    flop.flop_bench_force_tile_shape(-1)


SHAPES = list(range(14))
LAYERS = [(300, 200, 136, 264, 0), (333, 75, 41, 523, 8), (129, 264, 200, 72, 0), (70, 9, 3, 5, 8), (520, 1032, 72, 136, 0),
          (1, 64, 64, 64, 0), (257, 130, 258, 68, 8)]


def test_shape_table_matches_names():
    assert len(flop.flop_bench_tile_shapes()) == len(SHAPES)


@pytest.mark.parametrize("forced_shape", SHAPES, indirect=True)
@pytest.mark.parametrize("layer", LAYERS, ids=lambda s: "x".join(map(str, s[:4])))
def test_layer_with_forced_block_shape(forced_shape, layer):
    n, d, r, dout, align = layer
    check_layer(synth.layer_inputs(9800 + n + d, n, d, r, dout, "bf16"), align=align)


@pytest.mark.parametrize("forced_shape", SHAPES, indirect=True)
@pytest.mark.parametrize("case", ["single_layer_no_pending", "offsets_not_multiples_of_four", "four_aligned_layers"])
def test_riders_with_forced_block_shape(forced_shape, case):
    rider_step(case)
