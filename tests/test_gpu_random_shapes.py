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


def _draw(i):
    """A wider draw (added with the bf16 gate kernel for 17 to 256 experts): expert counts on both sides of every
    kernel's switching points (16 / 32 / 256 experts for the gate, 96 rows per expert for the tile shapes), one to
    eight experts per token, up to 6000 tokens."""
    g = np.random.default_rng([2103, 13262, i])
    E = int(g.choice([1, 2, 4, 6, 8, 10, 15, 16, 17, 31, 32, 33, 48, 64, 65, 100, 130, 256, 260]))
    k = int(g.integers(1, min(E, 8) + 1))
    d = 32 * int(g.integers(1, 17))
    h = 32 * int(g.choice([1, 2, 4, 7, 8, 16, 32, 64, 65, 128]))
    budget = 2.5e8 / (d * h * k)
    N = int(max(1, min(6000, g.integers(1, max(2, int(budget))))))
    zipf = float(g.choice([0.0, 0.5, 1.2]))
    dtype = "bf16" if i % 4 else "f32"
    return Workload(f"random_{i}", N, d, h, E, k, dtype, zipf, 7100 + i, 0.1 if i % 2 else 0.0, i % 3 == 1)


@pytest.mark.parametrize("i", range(32))
def test_wider_random_shape_matches_oracle(i):
    _full_check(_draw(i))
