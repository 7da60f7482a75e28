"""GPU parity of the eviction path against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest

from paper_2507_06517_amd import workloads as wl

import parity

pytestmark = pytest.mark.gpu


def test_config1_fp32(oracle):
    rep = parity.check_deep_layer(oracle, wl.config1(0))
    print("config1 deep", rep)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("l,lw,hn,pool,budget", [(300, 16, 4, 7, 64), (1000, 8, 2, 1, 200), (777, 64, 4, 15, 100),
                                                 (130, 32, 8, 3, 33), (65, 64, 1, 7, 64)])
def test_small_ragged(oracle, dtype, l, lw, hn, pool, budget):
    L = wl.small_random(3, dtype, B=2, H=2, l=l, hn=hn, lw=lw, pool=pool, budget=budget)
    parity.check_deep_layer(oracle, L)


@pytest.mark.parametrize("seed", range(12))
def test_shape_sweep(oracle, seed):
    # sequence lengths around the block and stage sizes of the kernels (128-key stages, 1024 keys
    # per block), every window x group size up to the limit of 256 rows, odd pooling widths
    rng = np.random.default_rng(2000 + seed)
    hn = int(rng.choice([1, 2, 4, 8]))
    lw = int(rng.choice([w for w in (1, 3, 16, 32, 64, 128, 256) if w * hn <= 256]))
    l = lw + int(rng.choice([0, 1, 127, 128, 129, 1023, 1024, 1025, 2047, 3000, 5000]))
    pool = int(rng.choice([1, 3, 7, 15, 31]))
    budget = int(rng.integers(lw, l + 2))
    dtype = ("f16", "bf16", "f32")[seed % 3]
    L = wl.small_random(200 + seed, dtype, B=1, H=2, l=l, hn=hn, lw=lw, pool=pool, budget=budget)
    rep = parity.check_deep_layer(oracle, L, norm=seed & 1)
    print("sweep", seed, dtype, l, lw, hn, pool, budget, rep, flush=True)


def test_norm_none_and_budget_edges(oracle):
    L = wl.small_random(4, "f16", B=1, H=2, l=600, hn=4, lw=32, pool=7, budget=100)
    parity.check_deep_layer(oracle, L, norm=1)
    for budget in (32, 33, 599, 600, 5000):       # window only, +1, all but one, all, more than all
        parity.check_deep_layer(oracle, L, budget=budget)


def test_zero_queries_closed_form():
    # Q = 0 makes every softmax row uniform: with the paper's divisor the last k context
    # tokens win, without it all tie and the first k win (lowest index).
    L = wl.small_random(5, "f16", B=1, H=1, l=700, hn=4, lw=16, pool=1, budget=116)
    L.Qw = np.zeros_like(L.Qw)
    lc = 700 - 16
    kept, _, _, sc = parity.gpu_deep(L, norm=0)
    assert kept[0, 0].tolist() == list(range(lc - 100, 700))
    h = sum(1.0 / (lc + b + 1) for b in range(16))
    np.testing.assert_allclose(sc[0, 0, :lc], h / (700 - np.arange(lc)), rtol=1e-5)
    kept, _, _, sc = parity.gpu_deep(L, norm=1)
    assert kept[0, 0].tolist() == list(range(100)) + list(range(lc, 700))


def test_per_unit_budgets(oracle):
    L = wl.small_random(6, "f16", B=2, H=2, l=500, hn=4, lw=16, pool=7, budget=64)
    budgets = [16, 64, 200, 500]
    kept, Ko, Vo, sc = parity.gpu_deep(L, budget=16, budgets=budgets, out_stride=500)
    for u, bud in enumerate(budgets):
        b, h = divmod(u, 2)
        one = wl.Layer(L.dtype, L.K[b:b + 1, h:h + 1], L.V[b:b + 1, h:h + 1], L.Qw[b:b + 1, 4 * h:4 * h + 4],
                       4, 16, 7, bud, 64)
        p64, k64 = parity.oracle_deep(oracle, one, bud)
        parity.check_deep_unit(p64[0, 0], k64[0, 0], sc[b, h], kept[b, h], 16, 500, {})


def test_config2(oracle):
    rep = parity.check_deep_layer(oracle, wl.config2(0))
    print("config2 deep", rep)


def test_deterministic_across_runs():
    L = wl.config2(1)
    a = parity.gpu_deep(L)
    b = parity.gpu_deep(L)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
