"""Parity at the full sizes of the benchmark configurations (configs 3-5), in the launch
configuration bench.py times.  The oracle runs on the host cores in parallel over units."""
import numpy as np
import pytest

from paper_2507_06517_amd import workloads as wl

import parity

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


@pytest.mark.parametrize("layers", [range(0, 4), range(4, 8)], ids=["0-3", "4-7"])
def test_config3_codebook_layers(oracle, layers):
    # 32-layer stack at l = 8192, layers 0-7: codebook replacement with cap 512.  Every layer goes
    # through the library and every one of its 16 problems is compared with the oracle.
    for layer in layers:
        L = wl.config3_layer(layer)
        assert L.max_codes == 512
        res, g = parity.check_shallow_layer(oracle, L, debug=layer in (0, 7))
        assert len(res) == 16
        print("config3 codebook layer", layer, [o["n_codes_uncapped"] for o in res][:4], flush=True)


@pytest.mark.parametrize("layers", [range(8, 16), range(16, 24), range(24, 32)], ids=["8-15", "16-23", "24-31"])
def test_config3_eviction_layers(oracle, layers):
    # layers 8-31: eviction with the budget tapering from 2048 to 256; all 8 units of every layer
    assert wl.config3_budget(8) == 2048 and wl.config3_budget(31) == 256
    rep = {}
    for layer in layers:
        L = wl.config3_layer(layer)
        assert L.budget == wl.config3_budget(layer)
        r = parity.check_deep_layer(oracle, L)
        if r:
            rep[layer] = r
    print("config3 eviction layers", list(layers), "selections inside the ambiguity band:", rep, flush=True)


def test_config3_stack_folded_into_batch(oracle):
    # layers folded into the batch dimension with per-unit budgets: one call for 4 layers
    layers = [8, 16, 24, 31]
    Ls = [wl.config3_layer(i, seq_len=2048) for i in layers]
    big = wl.Layer("f16", np.concatenate([x.K for x in Ls]), np.concatenate([x.V for x in Ls]),
                   np.concatenate([x.Qw for x in Ls]), 4, 32, 7, 2048, 512)
    budgets = [wl.config3_budget(i) for i in layers for _ in range(8)]
    kept, Ko, Vo, sc = parity.gpu_deep(big, budget=32, budgets=budgets, out_stride=2048)
    for j, L in enumerate(Ls):
        p64, k64 = parity.oracle_deep(oracle, L, L.budget)
        for h in range(8):
            parity.check_deep_unit(p64[0, h], k64[0, h], sc[j, h], kept[j, h], 32, 2048, {})


# the oracle's codebook results of the config-4 layer, shared by the tests that run it through
# different launch configurations (one computation of the 16 problems instead of three)
CONFIG4_ORACLE = {}


def test_config4_deep(oracle):
    rep = parity.check_deep_layer(oracle, wl.config4(0))
    print("config4 deep", rep, flush=True)


def test_config4_shallow(oracle):
    L = wl.config4(0)
    g = parity.gpu_shallow(L, debug=False)
    res, _ = parity.check_shallow_layer(oracle, L, g=g, cache=CONFIG4_ORACLE)
    print("config4 codes", [o["n_codes_uncapped"] for o in res], flush=True)


def test_config4_two_streams(oracle):
    # the eviction call on a side stream beside the second half of the codebook call (bench.py
    # --no-pipeline), run twice into the same buffers
    L = wl.config4(0)
    got, g = parity.gpu_layer_two_streams(L)
    rep = parity.check_deep_layer(oracle, L, got=got)
    res, _ = parity.check_shallow_layer(oracle, L, g=g, cache=CONFIG4_ORACLE)
    print("config4 on two streams", rep, [o["n_codes_uncapped"] for o in res][:4], flush=True)


def test_config4_pipelined(oracle):
    # the launch configuration bench.py times: consecutive steps pipelined over three sets of buffers.
    # Ten steps; the first set against the oracle in full, the others identical to the first
    L = wl.config4(0)
    (got0, g0), *others = parity.gpu_layers_pipelined(L, steps=10, depth=3)
    rep = parity.check_deep_layer(oracle, L, got=got0)
    res, _ = parity.check_shallow_layer(oracle, L, g=g0, cache=CONFIG4_ORACLE)
    assert len(others) == 2
    for got1, g1 in others:
        for a, b in zip(got0, got1):
            assert np.array_equal(a, b)
        for k in g0:
            assert np.array_equal(g0[k], g1[k]), k
    print("config4 pipelined", rep, [o["n_codes_uncapped"] for o in res][:4], flush=True)


def test_config4_adjacency_rows(oracle):
    # sampled rows of G and their degrees at l = 32768, every unit of K
    L = wl.config4(0)
    g = parity.gpu_shallow(L, tensors=("k",))
    rng = np.random.default_rng(0)
    theta = float(np.float32(L.theta_k))
    for h in range(L.n_kv_heads):
        X = wl.to_f64(L.K[0, h], L.dtype)
        m = oracle.magnitudes(X)
        for a in rng.integers(0, L.seq_len, size=24):
            row = oracle.adjacency_row(X, theta, int(a), m)
            assert np.array_equal(g["adj_k"][0, h, a], row)
            assert g["deg_k"][0, h, a] == sum(bin(int(w)).count("1") for w in row)


CONFIG5_CAPS = (512, 4096)


@pytest.fixture(scope="module")
def config5_on_gpu():
    """Layer -> ({cap: Layer}, {cap: library result of the codebook path}) of the batch-4 bf16
    stack, both caps of the sweep; one layer is held at a time."""
    held = {}

    def get(layer):
        if layer not in held:
            held.clear()
            Ls = {c: wl.config5_layer(layer, c) for c in CONFIG5_CAPS}
            L = Ls[CONFIG5_CAPS[0]]
            assert all(np.array_equal(Ls[c].K, L.K) and np.array_equal(Ls[c].V, L.V) for c in CONFIG5_CAPS)
            gs = {c: parity.gpu_shallow(Ls[c], debug=False) for c in CONFIG5_CAPS}
            for c in CONFIG5_CAPS:                     # invariants on every unit
                for t in ("k", "v"):
                    assert (gs[c][f"n_codes_{t}"] == c).all()
                    assert gs[c][f"ref_{t}"].min() >= 0 and gs[c][f"ref_{t}"].max() < c
            held[layer] = (Ls, gs)
        return held[layer]

    yield get
    held.clear()


@pytest.mark.parametrize("layer,part", [(0, "eviction"), (0, 0), (0, 1), (0, 2), (0, 3), (31, "eviction"), (31, "spread")])
def test_config5_layer(oracle, config5_on_gpu, layer, part):
    # batch 4 x 32768, bf16, pool 15, half of the tokens isolated noise; budgets and caps 512 and
    # 4096.  The whole layer runs on the GPU under both.
    # "eviction": every unit of the layer under both budgets.
    # Codebook path: every problem overflows both caps by far (some 12 k tokens lose their entry
    # and go through the cap step); the oracle builds the graph of a problem once and applies
    # both caps to it.  Layer 0: every (batch, head) problem of K and V, the 16 problems of one
    # batch entry per test case (one per host core); layer 31: one head of each batch entry.
    Ls, gs = config5_on_gpu(layer)
    if part == "eviction":
        for c in CONFIG5_CAPS:
            rep = parity.check_deep_layer(oracle, Ls[c])
            print("config5 layer", layer, "eviction, budget", c, rep, flush=True)
        return
    units = [(part, h) for h in range(8)] if part != "spread" else [(0, 5), (1, 2), (2, 7), (3, 0)]
    res = parity.check_shallow_layer_caps(oracle, Ls[CONFIG5_CAPS[0]], gs, units=units)
    assert len(res) == 2 * len(units)
    found = [o[CONFIG5_CAPS[0]]["n_codes_uncapped"] for (_, _, _, o) in res]
    assert min(found) > CONFIG5_CAPS[1], "every problem is meant to overflow both caps"
    print("config5 layer", layer, part, "codebook problems checked:", len(res), "entries found",
          min(found), "-", max(found), flush=True)


def test_max_seq_len_codebook(oracle):
    # the longest sequence the codebook path takes (token indices are 16 bits wide), with a
    # ragged last tile: sampled rows of G and their degrees against the oracle, then the
    # oracle's merge run on the library's G must give the library's codebook and references
    n = 65535
    L = wl.small_random(21, "f16", B=1, H=1, l=n, lw=1, cap=n, n_centroids=2000, noise_frac=0.1)
    g = parity.gpu_shallow(L, tensors=("k",))
    X = wl.to_f64(L.K[0, 0], L.dtype)
    theta = float(np.float32(L.theta_k))
    m = oracle.magnitudes(X)
    rng = np.random.default_rng(1)
    rows = [0, 1, 1023, 1024, 32767, 32768, 65472, n - 1] + rng.integers(0, n, size=24).tolist()
    for a in rows:
        row = oracle.adjacency_row(X, theta, int(a), m)
        assert np.array_equal(g["adj_k"][0, 0, a], row), f"row {a} of G differs"
        assert g["deg_k"][0, 0, a] == sum(bin(int(w)).count("1") for w in row)
    picks, ref = oracle.merge(g["adj_k"][0, 0])
    assert g["n_found_k"][0, 0] == len(picks) and g["n_codes_k"][0, 0] == len(picks)
    assert np.array_equal(g["ref_k"][0, 0], ref), "code assignment differs from the oracle's merge of the same G"
    assert np.array_equal(g["mag_k"][0, 0], m.astype(np.float32))
    parity.check_codebook_vectors(g["C_k"][0, 0, :len(picks)], X[picks] / m[picks, None], L.dtype)
    print("n = 65535:", len(picks), "codebook entries", flush=True)
    # without the adjacency output the lists come from the edge records instead of the bitmap:
    # same references and codebook as the run checked above
    g2 = parity.gpu_shallow(L, debug=False, tensors=("k",))
    assert g2["n_codes_k"][0, 0] == len(picks)
    assert np.array_equal(g2["ref_k"][0, 0], ref)
    assert np.array_equal(g2["C_k"][0, 0], g["C_k"][0, 0])


def test_long_ragged_deep(oracle):
    # a context longer than what the selection kernel keeps in LDS, not a multiple of any tile
    L = wl.small_random(22, "f16", B=1, H=2, l=100003, hn=4, lw=64, pool=7, budget=4096, cap=64, n_centroids=300)
    rep = parity.check_deep_layer(oracle, L)
    print("l = 100003 deep", rep, flush=True)
    L2 = wl.small_random(23, "bf16", B=1, H=1, l=40001, hn=4, lw=16, pool=15, budget=40001 - 5, cap=64, n_centroids=100)
    parity.check_deep_layer(oracle, L2)                 # nearly everything is kept


def test_eviction_then_codebook_on_the_kept_tokens(oracle):
    # composed use: the codebook is built over what the eviction kept (window included).  The
    # oracle selects rows with its own kept indices; the library works on its own gathered rows.
    L = wl.config2(0)
    p64, kept64 = parity.oracle_deep(oracle, L)
    kept, Ko, Vo, _ = parity.gpu_deep(L)
    B, H, l, d = L.K.shape
    assert np.array_equal(kept[..., :L.budget], kept64)
    kept_layer = wl.Layer(L.dtype, np.ascontiguousarray(Ko[:, :, :L.budget]),
                          np.ascontiguousarray(Vo[:, :, :L.budget]), L.Qw, L.group_size, L.window, L.pool,
                          L.budget, 256)
    g = parity.gpu_shallow(kept_layer, 256)
    for t, X, theta in (("k", L.K, L.theta_k), ("v", L.V, L.theta_v)):
        for h in range(H):
            X64 = wl.to_f64(X[0, h][kept64[0, h]], L.dtype)
            parity.check_shallow_unit(oracle, X64, theta, 256, L.dtype, g, t, 0, h)
    # Eq. 15 for this layer from the counts of both stages
    from paper_2507_06517_amd import binding as sb
    stored = int(g["n_codes_k"].sum() + g["n_codes_v"].sum())
    r1, r2, r3, r = sb.spindle_reserve_ratio(2 * H * L.budget, 2 * H * l, stored, d, 16, 16, 32)
    assert r1 == L.budget / l and 0 < r2 <= 256 / L.budget and abs(r - r1 * r2 * (d + 3) / d) < 1e-15
    assert np.array_equal(np.array([r1, r2, r3, r]), oracle.reserve_ratio(2 * H * L.budget, 2 * H * l, stored, d, 16, 16, 32))


def test_unfolded_gqa_then_one_codebook_per_kv_head(oracle):
    # The alternative for grouped-query models (Sec. "Attention Weight Based Token Eviction", last
    # paragraph): K and V are repeated once per query head, every query head evicts on its own
    # attention, and the codebook over the unfolded copies of a KV head removes the repetition
    # again (copies have cosine 1).  Both entry points are used as they are: the eviction with a
    # group size of one on the repeated tensors, the codebook on the concatenated kept rows.
    L = wl.config2(0)
    B, H, l, d = L.K.shape
    hn, budget, cap = L.group_size, 512, 640
    Kr, Vr = np.repeat(L.K, hn, axis=1), np.repeat(L.V, hn, axis=1)
    un = wl.Layer(L.dtype, Kr, Vr, L.Qw, 1, L.window, L.pool, budget, cap)
    p64, kept64 = parity.oracle_deep(oracle, un)
    kept, Ko, Vo, sc = parity.gpu_deep(un)
    rep = {}
    for q in range(H * hn):
        parity.check_deep_unit(p64[0, q], kept64[0, q], sc[0, q], kept[0, q], L.window, l, rep)
    assert not rep, "ambiguous selections would make the two codebooks start from different rows"
    folded = wl.Layer(L.dtype, np.ascontiguousarray(Ko[:, :, :budget]).reshape(B, H, hn * budget, d),
                      np.ascontiguousarray(Vo[:, :, :budget]).reshape(B, H, hn * budget, d), L.Qw, hn, L.window,
                      L.pool, budget, cap)
    g = parity.gpu_shallow(folded, cap)
    shared = []
    for t, X, theta in (("k", L.K, L.theta_k), ("v", L.V, L.theta_v)):
        for h in range(H):
            rows = np.concatenate([kept64[0, h * hn + j] for j in range(hn)])
            o = parity.check_shallow_unit(oracle, wl.to_f64(X[0, h][rows], L.dtype), theta, cap, L.dtype, g, t, 0, h)
            # copies of one token kept by several query heads end up in the same entry
            first = {}
            for pos, r in zip(rows, o["ref"]):
                assert first.setdefault(int(pos), int(r)) == int(r)
            shared.append(len(rows) - len(first))
    assert max(shared) > 0, "the query heads of a group should agree on some tokens"


def test_one_codebook_per_layer_over_the_unfolded_heads(oracle):
    # Sec. "Similarity Based Token Replacement", first paragraph, and Eq. 15's r_2: K and V repeated
    # once per query head, every query head evicts on its own attention (group size 1), and ONE
    # codebook per layer over the kept rows of all 32 heads removes the repetition again.  The
    # eviction outputs go into spindle_compress_shallow_layer as they are.
    import torch
    from paper_2507_06517_amd import binding as sb
    L = wl.config2(0)
    B, H, l, d = L.K.shape
    hn, budget, cap = L.group_size, 384, 1536
    Kr, Vr = np.repeat(L.K, hn, axis=1), np.repeat(L.V, hn, axis=1)
    un = wl.Layer(L.dtype, Kr, Vr, L.Qw, 1, L.window, L.pool, budget, cap)
    p64, kept64 = parity.oracle_deep(oracle, un)
    Kd, Vd, Qd = (sb.to_device(x, L.dtype) for x in (Kr, Vr, L.Qw))
    kept, Ko, Vo, sc = sb.compress_deep(Kd, Vd, Qd, 1, L.dtype, L.window, L.pool, budget, scale=parity.scale_of(d))
    torch.cuda.synchronize()
    assert np.array_equal(kept.cpu().numpy(), kept64), "the two codebooks must start from the same rows"
    out = sb.compress_shallow_layer(Ko, Vo, L.dtype, L.theta_k, L.theta_v, cap)
    torch.cuda.synchronize()
    g = {k: (sb.to_host_bits(v, L.dtype) if k.startswith("C_") else v.cpu().numpy()) for k, v in out.items() if k != "workspace"}
    Q = H * hn
    entries = 0
    for t, X, theta in (("k", L.K, L.theta_k), ("v", L.V, L.theta_v)):
        rows = np.concatenate([wl.to_f64(X[0, q // hn][kept64[0, q]], L.dtype) for q in range(Q)])
        assert rows.shape == (Q * budget, d)
        o = oracle.shallow_unit(rows, float(np.float32(theta)), cap)
        assert g[f"n_found_{t}"][0] == o["n_codes_uncapped"] and g[f"n_codes_{t}"][0] == o["n_codes"]
        assert np.array_equal(g[f"ref_{t}"][0].reshape(-1), o["ref"]), "code assignment differs"
        assert np.array_equal(g[f"mag_{t}"][0].reshape(-1), o["mag"].astype(np.float32))
        parity.check_codebook_vectors(g[f"C_{t}"][0, :o["n_codes"]], o["C"], L.dtype)
        assert not g[f"C_{t}"][0, o["n_codes"]:].any()
        # a token kept by several query heads of its KV head is one entry of the layer's codebook
        ref = g[f"ref_{t}"][0]
        shared = 0
        for h in range(H):
            first = {}
            for q in range(h * hn, (h + 1) * hn):
                for pos, r in zip(kept64[0, q], ref[q]):
                    shared += int(pos) in first
                    assert first.setdefault(int(pos), int(r)) == int(r)
        assert shared > 0
        entries += int(g[f"n_codes_{t}"][0])
        # per-head codebooks of the same rows need at least as many entries in total
        per_head = sum(oracle.shallow_unit(rows[q * budget:(q + 1) * budget], float(np.float32(theta)), cap)["n_codes"]
                       for q in range(0, Q, hn))
        assert o["n_codes_uncapped"] >= 1 and per_head >= 1
    # Eq. 15 with h_g = h (the repeat was made before the eviction): r_2 from the layer's two codebooks
    kept_rows, all_rows = 2 * Q * budget, 2 * Q * l
    r = sb.spindle_reserve_ratio(kept_rows, all_rows, entries, d, 16, 16, 32)
    assert np.array_equal(np.array(r), oracle.reserve_ratio(kept_rows, all_rows, entries, d, 16, 16, 32))
    assert r[0] == budget / l and r[1] == entries / kept_rows
    print("layer codebook over", Q * budget, "rows:", entries, "entries for K and V, r =", r, flush=True)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_cache_stored_token_major(oracle, dtype):
    # K and V kept as [batch, seq_len, heads, head_dim], the order many inference engines use:
    # the calls take the strides and read the rows in place.  Same results as the head-major copy.
    import torch
    from paper_2507_06517_amd import binding as sb
    L = wl.small_random(31, dtype, B=2, H=3, l=1300, hn=2, lw=16, pool=7, budget=200, cap=150, n_centroids=20)
    Kc, Vc, Q = (sb.to_device(x, L.dtype) for x in (L.K, L.V, L.Qw))
    Kt = Kc.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)          # [B, H, l, d] view of [B, l, H, d] memory
    Vt = Vc.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not Kt.is_contiguous() and torch.equal(Kt, Kc)
    kept, Ko, Vo, sc = sb.compress_deep(Kt, Vt, Q, L.group_size, L.dtype, L.window, L.pool, L.budget,
                                        scale=parity.scale_of(L.head_dim))
    torch.cuda.synchronize()
    p64, kept64 = parity.oracle_deep(oracle, L)
    rep = {}
    for b in range(2):
        for h in range(3):
            parity.check_deep_unit(p64[b, h], kept64[b, h], sc[b, h].cpu().numpy().astype(np.float64),
                                   kept[b, h].cpu().numpy(), L.window, 1300, rep)
            g = kept64[b, h]
            assert np.array_equal(sb.to_host_bits(Ko, dtype)[b, h, :len(g)], L.K[b, h][g])
            assert np.array_equal(sb.to_host_bits(Vo, dtype)[b, h, :len(g)], L.V[b, h][g])
    out = sb.compress_shallow(Kt, Vt, L.dtype, L.theta_k, L.theta_v, L.max_codes, debug=True)
    torch.cuda.synchronize()
    g = {}
    for k, v in out.items():
        g[k] = sb.to_host_bits(v, dtype) if k.startswith("C_") else (v.cpu().numpy().view(np.uint32) if k.startswith("adj_") else v.cpu().numpy())
    for t, X, theta in (("k", L.K, L.theta_k), ("v", L.V, L.theta_v)):
        for b in range(2):
            for h in range(3):
                parity.check_shallow_unit(oracle, wl.to_f64(X[b, h], dtype), theta, L.max_codes, dtype, g, t, b, h)
