"""Parity on seeded random shapes: the grouped products choose between whole tiles in rounds, tiles cut by rows and
tiles cut along the reduction from the tile counts, and the weight gradients between two ways of dealing tiles to
the XCDs, so a spread of shapes (expert counts that are no multiple of 8, reductions of 32 to 3072, skewed and
near-empty experts, top-1 to top-4, with and without expert biases, both score modes) walks through combinations that the named cases do not."""
import numpy as np
import pytest

from paper_2103_13262_amd.synth import Workload

from test_gpu_parity import _full_check

pytestmark = pytest.mark.gpu


def _shapes():
    g = np.random.default_rng(20210313)
    out = []
    for i in range(20):
        E = int(g.choice([1, 2, 3, 5, 7, 8, 9, 12, 16, 17, 24, 33, 40]))
        k = int(g.integers(1, min(E, 4) + 1))
        d = 32 * int(g.integers(1, 13))
        h = 32 * int(g.choice([1, 2, 3, 5, 8, 16, 33, 64, 96]))
        budget = 2.5e8 / (d * h * k)                      # keeps the fp64 oracle to a second or two
        N = int(max(1, min(2500, g.integers(1, max(2, int(budget))))))
        zipf = float(g.choice([0.0, 0.0, 0.8, 1.5]))
        dtype = "bf16" if i % 5 else "f32"
        out.append(Workload(f"rand{i}", N, d, h, E, k, dtype, zipf, 9000 + i, 0.1 if i % 3 == 0 else 0.0, i % 4 == 1))
    return out


@pytest.mark.parametrize("w", _shapes(), ids=lambda w: f"{w.name}-N{w.N}-d{w.d}-h{w.h}-E{w.E}-k{w.k}-{w.dtype}")
def test_random_shape_matches_oracle(w):
    _full_check(w)
