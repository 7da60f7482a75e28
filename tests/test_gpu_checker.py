"""Does the parity check look at every output?  One small layer goes through the HIP library
once; then one element of one output at a time is spoiled in a host copy and the comparison
with the oracle has to fail.  (The mistakes are planted in copies of the results on the host;
the kernels run once, unchanged.)"""
import copy

import numpy as np
import pytest

from paper_2507_06517_amd import workloads as wl

import parity

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]


def test_codebook_check_sees_every_output(oracle):
    L = wl.small_random(21, "f16", B=1, H=2, l=600, lw=1, cap=60, n_centroids=70, noise_frac=0.2)
    res, g = parity.check_shallow_layer(oracle, L)
    assert res[0]["n_codes_uncapped"] > 60                       # the cap is active: cut tokens exist
    nc = int(g["n_codes_k"][0, 1])

    def spoil(field, fn):
        bad = copy.deepcopy(g)
        fn(bad[field])
        with pytest.raises(AssertionError):
            parity.check_shallow_layer(oracle, L, g=bad)

    def flip_bit(a): a[0, 1, 300, 5] ^= np.uint32(1 << 7)
    def plus_one(a): a[0, 1, 17] += 1
    def count_up(a): a[0, 1] += 1
    def next_float(a): a[0, 1, 599] = np.nextafter(a[0, 1, 599], np.float32(np.inf))
    def nudge_entry(a): a[0, 1, nc - 1, 3] = (wl.to_f64(a[0, 1, nc - 1, 3:4], "f16") * 1.01 + 0.01).astype(np.float16)[0]
    def row_past_end(a): a[0, 1, nc, 0] = np.float16(1.0)

    for t in ("k", "v"):
        spoil(f"adj_{t}", flip_bit)
        spoil(f"deg_{t}", plus_one)
        spoil(f"ref_{t}", plus_one)
        spoil(f"mag_{t}", next_float)
        spoil(f"n_codes_{t}", count_up)
        spoil(f"n_found_{t}", count_up)
    spoil("C_k", nudge_entry)
    # and the unspoiled copy still passes
    parity.check_shallow_layer(oracle, L, g=copy.deepcopy(g))
    # rows past the stored entries (a table with room left)
    L = wl.small_random(23, "f16", B=1, H=2, l=300, lw=1, cap=300)
    res, g = parity.check_shallow_layer(oracle, L)
    nc = int(g["n_codes_k"][0, 1])
    assert nc < 300
    spoil("C_k", row_past_end)


def test_eviction_check_sees_every_output(oracle):
    L = wl.small_random(22, "f16", B=1, H=2, l=700, lw=16, budget=200)
    kept, Ko, Vo, sc = parity.gpu_deep(L)
    parity.check_deep_layer(oracle, L, got=(kept, Ko, Vo, sc))

    def spoil(i, fn):
        bad = [kept.copy(), Ko.copy(), Vo.copy(), sc.copy()]
        fn(bad[i])
        with pytest.raises(AssertionError):
            parity.check_deep_layer(oracle, L, got=tuple(bad))

    def other_token(a):
        free = np.setdiff1d(np.arange(700 - 16), a[0, 1])
        a[0, 1, 5] = free[np.searchsorted(free, a[0, 1, 5])]      # a neighbour that was not kept (order stays ascending or not: both must fail)
    def window_gone(a): a[0, 1, 199] = a[0, 1, 198]
    def padding(a): a[0, 0, 199] = -1
    def flip16(a):
        v = a[0, 1, 7:8, 100].view(np.uint16)
        v ^= np.uint16(1)
    def score_off(a): a[0, 1, 350] *= 1.01

    spoil(0, other_token)
    spoil(0, window_gone)
    spoil(0, padding)
    spoil(1, flip16)
    spoil(2, flip16)
    spoil(3, score_off)
