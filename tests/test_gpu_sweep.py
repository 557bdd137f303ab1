"""Seeded sweep over shapes the other GPU tests do not visit: widths from 4 to 1024 (all three
register layouts of the row kernels, ragged tiles of the contraction kernel), hidden widths from
4 to 800, batch sizes from 1, K from 1, small and large margins; both operator families.
Same bars as tests/parity.py (needs an MI355X)."""
import numpy as np
import pytest

from tests import parity as par
from tests import parity_box as pb

pytestmark = pytest.mark.gpu


def shapes(seed):
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.choice([4, 8, 20, 36, 64, 100, 132, 256, 260, 400, 512, 516, 1024]))
    h = int(rng.choice([4, 12, 64, 72, 200, 800]))
    N, R = int(rng.integers(50, 3000)), int(rng.integers(2, 40))
    B, K = int(rng.integers(1, 120)), int(rng.integers(1, 40))
    return N, R, d, h, B, K, float(rng.uniform(2, 30))


@pytest.mark.parametrize("block", range(4))
def test_shape_sweep_both_families(block):
    for seed in range(4 * block, 4 * block + 4):
        N, R, d, h, B, K, gamma = shapes(seed)
        par.say("sweep %d: N=%d R=%d d=%d h=%d B=%d K=%d gamma=%.1f, both families" % (seed, N, R, d, h, B, K, gamma))
        vec = par.Case(N, R, d, h, B, K, gamma, seed=100 + seed)
        par.check_forward_backward(vec)
        box = pb.BoxCase(N, R, d, h, B, K, gamma / 4, alpha=0.1, seed=200 + seed,
                         schedule="max_fill" if seed % 2 else "level", b_max=(seed % 3) * 7)
        pb.check_forward_backward(box)
        if seed % 4 == 1:
            par.check_train_steps(vec, steps=2, num_streams=2)
            pb.check_train_steps(box, steps=2, num_streams=2)
