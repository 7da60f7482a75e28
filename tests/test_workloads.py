"""The synthetic generators: deterministic, exact dtype round trips, planted structure."""
import numpy as np
import torch

from paper_2507_06517_amd import workloads as wl


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(10000).astype(np.float32) * 10
    x[:4] = [0.0, -0.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8]      # exact ties round to even
    bits = wl.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    back = wl.to_f64(bits, "bf16")
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy())


def test_casts_are_exact_in_f64():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(1000)
    for dt in ("f32", "f16", "bf16"):
        bits = wl.cast(x, dt)
        v = wl.to_f64(bits, dt)
        assert np.array_equal(wl.to_f64(wl.cast(v, dt), dt), v)


def test_config1_structure_and_determinism():
    a, b = wl.config1(0), wl.config1(0)
    assert np.array_equal(a.K, b.K) and np.array_equal(a.Qw, b.Qw)
    assert a.K.shape == (1, 1, 512, 128) and a.Qw.shape == (1, 4, 32, 128) and a.dtype == "f32"
    planted, src = a.meta["planted"], a.meta["src"]
    assert planted.sum() == 128
    K = a.K[0, 0].astype(np.float64)
    Kn = K / np.linalg.norm(K, axis=1, keepdims=True)
    c = np.einsum("ad,ad->a", Kn[planted], Kn[src[planted]])
    assert c.min() > 0.984 and c.max() < 0.9995
    assert np.all(src[planted] < np.flatnonzero(planted))
    assert not np.array_equal(wl.config1(1).K, a.K)


def test_config2_shapes_and_cluster_cosines():
    L = wl.config2(0)
    assert L.K.shape == (1, 8, 4096, 128) and L.Qw.shape == (1, 32, 32, 128) and L.K.dtype == np.float16
    K = L.K[0, 3].astype(np.float64)
    a = L.meta["assign"][0, 3]
    Kn = K / np.linalg.norm(K, axis=1, keepdims=True)
    S = Kn[:300] @ Kn[:300].T
    same = a[:300, None] == a[None, :300]
    assert S[same].min() > 0.975 and np.median(S[same]) > 0.988 and np.abs(S[~same]).max() < 0.6
    norms = np.linalg.norm(K, axis=1)
    assert 0.02 < (norms > 30).mean() < 0.09                       # ~5 % heavy hitters at 4x norm


def test_config3_budgets_taper():
    b = [wl.config3_budget(i) for i in range(8, 32)]
    assert b[0] == 2048 and b[-1] == 256 and all(x >= y for x, y in zip(b, b[1:]))


def test_decode_case_mixes_known_and_new_directions():
    pre, new = wl.decode_case(1, "f16", B=1, H=2, n_prefill=300, m=96, novel_frac=0.3)
    assert pre.shape == (1, 2, 300, 128) and new.shape == (1, 2, 96, 128) and pre.dtype == np.float16
    pre2, new2 = wl.decode_case(1, "f16", B=1, H=2, n_prefill=300, m=96, novel_frac=0.3)
    assert np.array_equal(pre, pre2) and np.array_equal(new, new2)
    P, N = wl.to_f64(pre[0, 0], "f16"), wl.to_f64(new[0, 0], "f16")
    P /= np.linalg.norm(P, axis=1, keepdims=True)
    N /= np.linalg.norm(N, axis=1, keepdims=True)
    near = (N @ P.T).max(axis=1) > 0.98
    assert 0.5 < near.mean() < 0.85          # most later tokens resemble a prefill token, the novel ones none
