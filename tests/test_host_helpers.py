"""Host helpers of the library (layer budgets, reserve ratio) against the oracle and closed forms.
No GPU: the helpers are plain host arithmetic inside libspindle.so."""
import numpy as np
import pytest


@pytest.fixture(scope="module")
def sb():
    from paper_2507_06517_amd import binding
    binding.lib()
    return binding


def test_layer_budgets_match_oracle_ratios(sb, oracle):
    # Eq. 5-6: all three regimes (flat, floor at beta, ceiling at 1) and the knee itself
    l, lw, m, beta = 32768, 64, 32, 0.05
    lc = l - lw
    for rc in [0.02, 0.05, 0.2, 0.5, 0.525, 0.526, 0.8, 1.0]:
        r = (rc * lc + lw) / l
        budgets, ratios = sb.spindle_layer_budgets(r, l, lw, m, beta)
        want = oracle.layer_ratios(r, l, lw, m, beta)
        assert np.allclose(ratios, want, rtol=0, atol=1e-12)
        # Eq. 7: k = floor(r_c(layer) l_c); the oracle's own integers, not a formula of this test
        assert np.array_equal(budgets, oracle.layer_budgets(r, l, lw, m, beta))
        # the mean over layers stays at r_c: flooring loses less than one token per layer
        assert 0 <= m * r * l - int(budgets.sum()) < m + 1e-6
        assert np.all(np.diff(budgets) <= 0) and budgets.min() >= lw and budgets.max() <= l


def test_layer_budgets_printed_alpha_and_endpoints(sb):
    # beta = 0.05 gives alpha = 0.525 (the value the paper's text implies); at r_c = alpha the
    # first layer keeps everything and the last keeps beta
    l, lw, m = 10064, 64, 5
    lc = l - lw
    budgets, ratios = sb.spindle_layer_budgets((0.525 * lc + lw) / l, l, lw, m, 0.05)
    assert abs(ratios[0] - 1.0) < 1e-12 and abs(ratios[-1] - 0.05) < 1e-12
    assert budgets[0] in (l - 1, l) and budgets[-1] in (lw + 499, lw + 500)     # floor of a product within an ulp of an integer
    # linear in between (Eq. 6)
    assert np.allclose(np.diff(ratios), (0.05 - 1.0) / 4)
    # one layer: the mean itself
    b1, r1 = sb.spindle_layer_budgets(0.3, 1000, 100, 1, 0.05)
    assert abs(r1[0] - (300 - 100) / 900) < 1e-12 and b1[0] in (299, 300)


def test_layer_budgets_floor_as_printed(sb, oracle):
    # Eq. 7 floors: ratios chosen so that r_c(layer) l_c has fractional parts on both sides of
    # one half; rounding to nearest would differ from the expected integers written out here
    l, lw, m, beta = 1032, 32, 3, 0.05          # l_c = 1000
    # r_c = 0.3007: first = 0.5514, last = 0.05, middle = 0.3007 -> 551.4, 300.7, 50.0
    r = (0.3007 * 1000 + lw) / l
    budgets, ratios = sb.spindle_layer_budgets(r, l, lw, m, beta)
    assert abs(ratios[0] - 0.5514) < 1e-9 and abs(ratios[1] - 0.3007) < 1e-9
    assert budgets[0] == lw + 551 and budgets[1] == lw + 300
    assert np.array_equal(budgets, oracle.layer_budgets(r, l, lw, m, beta))
    # a sweep of ratios and shapes: the library's integers are the oracle's everywhere
    rng = np.random.default_rng(5)
    for _ in range(300):
        l = int(rng.integers(200, 70000))
        lw = int(rng.integers(1, 129))
        m = int(rng.integers(1, 81))
        beta = float(rng.choice([0.0, 0.05, 0.1, 0.3]))
        r = float(rng.uniform(lw / l, 1.0))
        budgets, _ = sb.spindle_layer_budgets(r, l, lw, m, beta)
        assert np.array_equal(budgets, oracle.layer_budgets(r, l, lw, m, beta)), (r, l, lw, m, beta)


def test_layer_budgets_reject_bad_arguments(sb):
    for args in [(0.5, 100, 0, 4, 0.05), (0.5, 100, 200, 4, 0.05), (0.5, 100, 10, 0, 0.05),
                 (1.5, 100, 10, 4, 0.05), (0.5, 100, 10, 4, -0.1)]:
        with pytest.raises(sb.SpindleError) as e:
            sb.spindle_layer_budgets(*args)
        assert e.value.code == 1


def test_reserve_ratio(sb, oracle):
    # Eq. 15 by hand: 1024 of 4096 tokens kept, 256 entries, 16-bit index and elements, d_h = 128
    # and a magnitude as wide as an element: the "+ 1" of the printed r3
    r = sb.spindle_reserve_ratio(1024, 4096, 256, 128, 16, 16, 16)
    assert r == (0.25, 0.25, 130 / 128, 0.25 * 0.25 * 130 / 128)
    assert np.array_equal(np.array(r), oracle.reserve_ratio(1024, 4096, 256, 128, 16, 16, 16))
    # the float32 magnitudes the library writes count as two 16-bit elements
    r = sb.spindle_reserve_ratio(1024, 4096, 256, 128, 16, 16, 32)
    assert r[2] == 131 / 128 and np.array_equal(np.array(r), oracle.reserve_ratio(1024, 4096, 256, 128, 16, 16, 32))
    # 32-bit index next to 16-bit elements counts as two elements
    assert sb.spindle_reserve_ratio(10, 10, 10, 64, 32, 16, 16)[2] == 67 / 64
    # float32 cache: index of half an element, magnitude of one
    assert sb.spindle_reserve_ratio(10, 10, 10, 128, 16, 32, 32)[2] == 129.5 / 128
    with pytest.raises(sb.SpindleError):
        sb.spindle_reserve_ratio(10, 5, 1)
    with pytest.raises(sb.SpindleError):
        sb.spindle_reserve_ratio(10, 20, 11)
