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
        assert np.array_equal(budgets, lw + np.floor(want * lc + 0.5).astype(np.int64))
        # the mean over layers stays at r_c: the total budget is the requested one up to rounding
        assert abs(int(budgets.sum()) - m * r * l) <= m
        assert np.all(np.diff(budgets) <= 0) and budgets.min() >= lw and budgets.max() <= l


def test_layer_budgets_printed_alpha_and_endpoints(sb):
    # beta = 0.05 gives alpha = 0.525 (the value the paper's text implies); at r_c = alpha the
    # first layer keeps everything and the last keeps beta
    l, lw, m = 10064, 64, 5
    lc = l - lw
    budgets, ratios = sb.spindle_layer_budgets((0.525 * lc + lw) / l, l, lw, m, 0.05)
    assert abs(ratios[0] - 1.0) < 1e-12 and abs(ratios[-1] - 0.05) < 1e-12
    assert budgets[0] == l and budgets[-1] == lw + 500
    # linear in between (Eq. 6)
    assert np.allclose(np.diff(ratios), (0.05 - 1.0) / 4)
    # one layer: the mean itself
    b1, r1 = sb.spindle_layer_budgets(0.3, 1000, 100, 1, 0.05)
    assert abs(r1[0] - (300 - 100) / 900) < 1e-12 and b1[0] == 300


def test_layer_budgets_reject_bad_arguments(sb):
    for args in [(0.5, 100, 0, 4, 0.05), (0.5, 100, 200, 4, 0.05), (0.5, 100, 10, 0, 0.05),
                 (1.5, 100, 10, 4, 0.05), (0.5, 100, 10, 4, -0.1)]:
        with pytest.raises(sb.SpindleError) as e:
            sb.spindle_layer_budgets(*args)
        assert e.value.code == 1


def test_reserve_ratio(sb, oracle):
    # Eq. 15 by hand: 1024 of 4096 tokens kept, 256 entries, 16-bit index and elements, d_h = 128
    r = sb.spindle_reserve_ratio(1024, 4096, 256, 128, 16, 16)
    assert r == (0.25, 0.25, 130 / 128, 0.25 * 0.25 * 130 / 128)
    assert np.array_equal(np.array(r), oracle.reserve_ratio(1024, 4096, 256, 128, 16, 16))
    # 32-bit index next to 16-bit elements counts as two elements
    assert sb.spindle_reserve_ratio(10, 10, 10, 64, 32, 16)[2] == 67 / 64
    with pytest.raises(sb.SpindleError):
        sb.spindle_reserve_ratio(10, 5, 1)
    with pytest.raises(sb.SpindleError):
        sb.spindle_reserve_ratio(10, 20, 11)
