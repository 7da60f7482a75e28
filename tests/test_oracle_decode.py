"""Pins of the oracle's decode-time merge (paragraph after Eq. 14): a hand-worked example,
reductions to Alg. 1 and to a closed form, and a dense numpy evaluation."""
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def _hand():
    rows = {}
    for line in open(os.path.join(HERE, "golden", "decode_hand.txt")):
        if line.startswith("#") or "|" not in line:
            continue
        k, v = line.split("|")
        rows[k.strip()] = v.split()
    return rows


def _dirs(deg):
    a = np.deg2rad(np.asarray(deg, dtype=np.float64))
    return np.stack([np.cos(a), np.sin(a)], axis=1)


def test_hand_worked_example(oracle):
    h = _hand()
    Cb = _dirs([float(x) for x in h["entries"]])
    ang, mag = zip(*[(float(t.split(":")[0]), float(t.split(":")[1])) for t in h["tokens"]])
    X = _dirs(ang) * np.array(mag)[:, None]
    for literal in (False, True):
        o = oracle.decode_merge(X, Cb, 0.95, 64, literal=literal)
        assert o["ref"].tolist() == [int(x) for x in h["ref"]]
        assert o["n_found"] == int(h["found"][0]) and o["n_codes"] == o["n_found"]
        assert o["n_matched"] == int(h["matched"][0])
        np.testing.assert_allclose(o["mag"], mag, rtol=1e-15)
        np.testing.assert_allclose(o["C_new"], _dirs([float(x) for x in h["new"]]), atol=1e-15)
    o = oracle.decode_merge(X, Cb, 0.95, 6)
    assert o["ref"].tolist() == [int(x) for x in h["ref_cap6"]]
    assert o["n_found"] == 7 and o["n_codes"] == 6 and o["C_new"].shape[0] == 1


def _clustered(rng, n, d, k, noise):
    cent = rng.standard_normal((k, d))
    return cent[rng.integers(0, k, n)] + noise * rng.standard_normal((n, d))


def test_empty_codebook_is_alg1(oracle):
    rng = np.random.default_rng(5)
    X = _clustered(rng, 150, 16, 9, 0.12)
    ref = oracle.shallow_unit(X, 0.9, 1000)
    o = oracle.decode_merge(X, np.zeros((0, 16)), 0.9, 1000)
    assert o["n_matched"] == 0 and o["n_found"] == ref["n_codes_uncapped"]
    assert np.array_equal(o["ref"], ref["ref"]) and np.array_equal(o["C_new"], ref["C"])
    assert np.array_equal(o["mag"], ref["mag"])


def test_scaled_copies_of_entries_all_merge(oracle):
    rng = np.random.default_rng(6)
    Cb = rng.standard_normal((12, 8))
    Cb /= np.linalg.norm(Cb, axis=1, keepdims=True)
    which = rng.integers(0, 12, 40)
    scale = rng.uniform(0.5, 4.0, 40)
    o = oracle.decode_merge(Cb[which] * scale[:, None], Cb, 0.98, 12)
    assert o["n_matched"] == 40 and o["n_found"] == 12 and o["C_new"].shape[0] == 0
    assert np.array_equal(o["ref"], which)
    np.testing.assert_allclose(o["mag"], scale, rtol=1e-14)
    # the cosine of Eq. 4 divides by the stored row's own norm: rows that are not of unit length
    # (as after rounding to the storage type, here grossly) give the same matches
    stretch = rng.uniform(0.25, 3.0, 12)
    o2 = oracle.decode_merge(Cb[which] * scale[:, None], Cb * stretch[:, None], 0.98, 12)
    assert o2["n_matched"] == 40 and np.array_equal(o2["ref"], which)


def test_against_dense_numpy(oracle):
    rng = np.random.default_rng(7)
    for theta in (0.9, 0.5, -1.0):
        d = 24
        base = _clustered(rng, 300, d, 14, 0.15)
        pre = oracle.shallow_unit(base[:200], theta if theta > 0 else 0.9, 1000)
        Cb = pre["C"].astype(np.float32).astype(np.float64)          # stored rows are rounded
        X = base[200:]
        o = oracle.decode_merge(X, Cb, theta, 1000)
        S = (X @ Cb.T) / np.outer(np.linalg.norm(X, axis=1), np.linalg.norm(Cb, axis=1))
        assert np.abs(S - theta).min() > 1e-9, "a cosine sits on the threshold: pick another seed"
        srt = np.sort(S, axis=1)
        assert (srt[:, -1] - srt[:, -2]).min() > 1e-9, "two entries tie: pick another seed"
        want = np.where(S.max(axis=1) > theta, S.argmax(axis=1), -1)
        matched = want >= 0
        assert np.array_equal(o["ref"][matched], want[matched]) and o["n_matched"] == matched.sum()
        if theta == -1.0:
            assert matched.all()
        rest = oracle.shallow_unit(X[~matched], theta, 1000) if (~matched).any() else None
        if rest is not None:
            assert np.array_equal(o["ref"][~matched], len(Cb) + rest["ref"])
            assert np.array_equal(o["C_new"], rest["C"])
            assert o["n_found"] == len(Cb) + rest["n_codes_uncapped"]
        # every token is within theta of the direction that replaces it
        full = np.concatenate([Cb, o["C_new"]])
        rec = full[o["ref"]]
        cs = np.einsum("ij,ij->i", rec, X) / (np.linalg.norm(rec, axis=1) * np.linalg.norm(X, axis=1))
        assert (cs > theta).all()


def test_zero_vectors_and_no_new_tokens_of_note(oracle):
    Cb = np.eye(4)
    X = np.zeros((3, 4))
    X[1] = [0, 2, 0, 0]
    o = oracle.decode_merge(X, Cb, 0.9, 10)
    # a zero vector has cosine 0 with everything: unmatched, and each is its own (zero) entry
    assert o["ref"].tolist() == [4, 1, 5] and o["n_found"] == 6
    assert not o["C_new"].any() and o["mag"].tolist() == [0.0, 2.0, 0.0]


def test_threshold_is_strict(oracle):
    # a 3-4-5 triangle: cos((4, 3), (1, 0)) = 4 / 5, the same double as the literal 0.8.  Eq. 9 is a
    # strict comparison, so at theta = 0.8 the token does not merge and founds an entry of its own
    Cb = np.array([[1.0, 0.0, 0.0, 0.0]])
    X = np.array([[4.0, 3.0, 0.0, 0.0]])
    assert 4.0 / (5.0 * 1.0) == 0.8
    o = oracle.decode_merge(X, Cb, 0.8, 8)
    assert o["n_matched"] == 0 and o["ref"].tolist() == [1] and o["n_found"] == 2
    np.testing.assert_allclose(o["C_new"], [[0.8, 0.6, 0.0, 0.0]], rtol=1e-15)
    o = oracle.decode_merge(X, Cb, np.nextafter(0.8, 0.0), 8)
    assert o["n_matched"] == 1 and o["ref"].tolist() == [0] and o["n_found"] == 1
