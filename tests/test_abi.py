"""The C-ABI library loads, exports every symbol the header declares, and its host-side
validation returns error codes without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sb():
    from paper_2507_06517_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2507_06517_amd import build
        build.build_library(verbose=False)
    binding.lib()
    return binding


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in os.listdir(inc):
        if f.endswith(".h"):
            text = open(os.path.join(inc, f)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(spindle_[a-z_]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported(sb):
    names = declared_symbols()
    assert {"spindle_compress_deep", "spindle_compress_shallow", "spindle_reconstruct",
            "spindle_deep_workspace_bytes", "spindle_shallow_workspace_bytes"} <= names
    L = sb.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert set(sb.EXPORTS) == names
    assert L.spindle_version() >= 1


def test_workspace_queries_and_validation(sb):
    d = sb.KvDesc(1, 8, 4, 32768, 128, sb.F16)
    deep = sb.spindle_deep_workspace_bytes(d, 64)
    assert 0 < deep < 64 << 20
    sh = sb.spindle_shallow_workspace_bytes(d, 2)
    assert sh >= 16 * 32768 * 32768 // 8            # dominated by the adjacency bits
    assert sb.spindle_shallow_workspace_bytes(d, 1) < sh
    bad = [
        (sb.KvDesc(1, 8, 4, 4096, 64, sb.F16), 32, 2),     # head_dim
        (sb.KvDesc(0, 8, 4, 4096, 128, sb.F16), 32, 1),    # batch
        (sb.KvDesc(1, 8, 4, 4096, 128, 7), 32, 1),         # dtype
        (sb.KvDesc(1, 8, 4, 4096, 128, sb.F16), 0, 1),     # window
        (sb.KvDesc(1, 8, 4, 4096, 128, sb.F16), 5000, 1),  # window > seq_len
        (sb.KvDesc(1, 8, 8, 4096, 128, sb.F16), 64, 2),    # window * group_size > 256
    ]
    for desc, window, code in bad:
        with pytest.raises(sb.SpindleError) as e:
            sb.spindle_deep_workspace_bytes(desc, window)
        assert e.value.code == code and str(e.value)
    with pytest.raises(sb.SpindleError) as e:
        sb.spindle_shallow_workspace_bytes(sb.KvDesc(1, 1, 1, 70000, 128, sb.F16), 1)
    assert e.value.code == 2
    with pytest.raises(sb.SpindleError):
        sb.spindle_shallow_workspace_bytes(d, 3)


def test_compress_calls_reject_bad_arguments_before_any_launch(sb):
    L = sb.lib()
    d = sb.KvDesc(1, 2, 4, 512, 128, sb.F16)
    fake = C.c_void_p(0x1000)       # never dereferenced: validation fails first
    null = C.c_void_p(0)

    def deep(**kw):
        a = dict(K=fake, V=fake, Qw=fake, window=32, pool=7, scale=0.088, norm=0, budget=128, budgets=null,
                 out_stride=128, kept=fake, Ko=fake, Vo=fake, sc=null, ws=fake, wsb=1 << 30)
        a.update(kw)
        return L.spindle_compress_deep(C.byref(a.get("desc", d)), a["K"], a["V"], a["Qw"], a["window"], a["pool"], a["scale"],
                                       a["norm"], a["budget"], a["budgets"], a["out_stride"], a["kept"],
                                       a["Ko"], a["Vo"], a["sc"], a["ws"], a["wsb"], null)

    assert deep(K=null) == 1
    assert deep(pool=4) == 1
    assert deep(pool=0) == 1
    assert deep(norm=3) == 1
    assert deep(budget=16) == 1
    assert deep(out_stride=64) == 1
    assert deep(Vo=null) == 1
    assert deep(scale=float("nan")) == 1
    assert deep(ws=null) == 3
    assert deep(wsb=16) == 3
    assert deep(ws=C.c_void_p(0x1010)) == 3
    assert deep(K=C.c_void_p(0x1004)) == 1
    assert b"aligned" in L.spindle_last_error()
    # strides of K and V: token stride below head_dim, not a multiple of 8 elements, negative
    assert deep(desc=sb.KvDesc(1, 2, 4, 512, 128, sb.F16, 0, 0, 64)) == 1
    assert deep(desc=sb.KvDesc(1, 2, 4, 512, 128, sb.F16, 0, 132, 0)) == 1
    assert deep(desc=sb.KvDesc(1, 2, 4, 512, 128, sb.F16, -256, 0, 0)) == 1

    def shallow(**kw):
        a = dict(K=fake, V=null, cap=64, C=fake, nc=fake, ref=fake, mag=fake, ws=fake, wsb=1 << 40, tk=0.98)
        a.update(kw)
        return L.spindle_compress_shallow(C.byref(d), a["K"], a["V"], a["tk"], 0.95, a["cap"], a["C"], null, a["nc"],
                                          null, null, null, a["ref"], null, a["mag"], null, null, null, null, null,
                                          a["ws"], a["wsb"], null)

    assert shallow(K=null) == 1
    assert shallow(cap=0) == 1
    # the two halves of the call validate the same way
    for half in (L.spindle_shallow_graph, L.spindle_shallow_codebook):
        assert half(C.byref(d), null, null, 0.98, 0.95, 64, fake, null, fake, null, null, null, fake, null, fake,
                    null, null, null, null, null, fake, 1 << 40, null) == 1
        assert half(C.byref(d), fake, null, 0.98, 0.95, 64, fake, null, fake, null, null, null, fake, null, fake,
                    null, null, null, null, null, fake, 1024, null) == 3
    assert shallow(ref=null) == 1
    assert shallow(tk=float("nan")) == 1
    assert shallow(wsb=1024) == 3
    assert L.spindle_reconstruct(1, 16, 64, sb.F16, 4, fake, fake, fake, fake, null) == 2
    assert L.spindle_reconstruct(1, 16, 128, sb.F16, 4, null, fake, fake, fake, null) == 1

    # decode-time merge: validation happens before anything is enqueued
    dd = sb.KvDesc(1, 2, 1, 64, 128, sb.F16)

    def decode(**kw):
        a = dict(d=dd, X=fake, th=0.98, cap=16, C=fake, nc=fake, nf=fake, ref=fake, mag=fake, ws=fake, wsb=1 << 20)
        a.update(kw)
        return L.spindle_decode_merge(C.byref(a["d"]), a["X"], a["th"], a["cap"], a["C"], a["nc"], a["nf"], null,
                                      a["ref"], a["mag"], a["ws"], a["wsb"], null)

    assert decode(X=null) == 1
    assert decode(cap=0) == 1
    assert decode(th=1.0) == 1
    assert decode(wsb=16) == 3
    assert decode(d=sb.KvDesc(1, 2, 1, 1025, 128, sb.F16)) == 2
    assert decode(d=sb.KvDesc(1, 2, 1, 64, 64, sb.F16)) == 2
    assert sb.spindle_decode_workspace_bytes(dd, 16) >= 2 * 64 * 8 * 129


def test_missing_library_raises_instead_of_falling_back(sb, monkeypatch, tmp_path):
    # there is no CPU path: without the built library every product call must fail loudly
    monkeypatch.setattr(sb, "_lib", None)
    monkeypatch.setattr(sb, "LIB_PATH", str(tmp_path / "libspindle.so"))
    with pytest.raises(FileNotFoundError):
        sb.lib()
    with pytest.raises(FileNotFoundError):
        sb.spindle_deep_workspace_bytes(sb.KvDesc(1, 8, 4, 4096, 128, sb.F16), 32)
    with pytest.raises(FileNotFoundError):
        sb.spindle_layer_budgets(0.5, 4096, 32, 8)


def test_layer_codebook_shape_limits(sb):
    # one codebook over all heads of a layer = one problem of heads x tokens rows
    d = sb.KvDesc(2, 32, 1, 2047, 128, sb.F16)                 # 65504 rows: the largest unfolded layer with 32 heads
    one = sb.KvDesc(2, 1, 1, 32 * 2047, 128, sb.F16)
    assert sb.spindle_shallow_layer_workspace_bytes(d, 2) == sb.spindle_shallow_workspace_bytes(one, 2)
    with pytest.raises(sb.SpindleError) as e:
        sb.spindle_shallow_layer_workspace_bytes(sb.KvDesc(1, 32, 1, 2048, 128, sb.F16), 1)    # 65536 rows
    assert e.value.code == 2 and "65535" in str(e.value) and "65536" in str(e.value)
    # a token-major cache ([B, l, H, d]) does not have the heads of a batch entry one behind the other
    with pytest.raises(sb.SpindleError) as e:
        sb.spindle_shallow_layer_workspace_bytes(sb.KvDesc(1, 8, 1, 512, 128, sb.F16, 8 * 512 * 128, 128, 8 * 128), 1)
    assert e.value.code == 2 and "follow each other" in str(e.value)
    # head-major with padding between batch entries is fine
    assert sb.spindle_shallow_layer_workspace_bytes(sb.KvDesc(2, 8, 1, 512, 128, sb.F16, 9 * 512 * 128, 512 * 128, 128), 1) > 0
