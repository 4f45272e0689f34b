"""GPU parity on seeded random shapes: sequence counts and lengths, GQA ratios, block
sizes and per-(sequence, head) budgets drawn at random, every case through the whole
path and compared with the oracle like the hand-picked cases."""
import numpy as np
import pytest

from workloads import make_custom

from test_gpu_parity import full_parity

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(8))
def test_random_shape(seed):
    rng = np.random.default_rng(7000 + seed)
    block = int(rng.choice([64, 128]))
    n_seq = int(rng.integers(1, 5))
    seqlens = [int(rng.integers(1, 12 * block)) for _ in range(n_seq)]
    hkv = int(rng.choice([1, 2, 4]))
    hq = hkv * int(rng.choice([1, 2, 4, 8]))
    hq = min(hq, 16)
    hkv = hq // max(1, hq // hkv)
    nb_max = max(-(-s // block) for s in seqlens)
    budgets = rng.integers(0, nb_max + 3, size=n_seq * hq).tolist()      # 0 and 1 are raised to 2, large ones clipped
    wl = make_custom(seqlens, hq, hkv, block, budgets, seed=7100 + seed, name="random%d" % seed)
    run = full_parity(wl)
    st = run.stats_host()
    assert st["n_items"].sum() == run.rows and st["cost_blocks"].sum() == run.sel_ptr_host[-1]
