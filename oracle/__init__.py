"""ctypes wrapper around the CPU oracle (``spindle_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``; never by the product path.
It shares nothing with the HIP library.  All arithmetic is in the C file;
this module only marshals numpy arrays (float64 values of the device tensors).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spindle_oracle.c")
# SPINDLE_ORACLE_LIB: load this library instead (the mutation check of the pins compiles deliberately
# broken copies of the C file and runs the pin tests against them).
_OVERRIDE = os.environ.get("SPINDLE_ORACLE_LIB")
_LIB = _OVERRIDE or os.path.join(_HERE, "libspindle_oracle.so")
_lib = None

_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(dtype=np.uint32, flags="C_CONTIGUOUS")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math: summation order is part of its definition)."""
    if _OVERRIDE:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.oracle_deep_scores.argtypes = [_f64p, _f64p, C.c_int, C.c_int, C.c_int, C.c_int,
                                         C.c_double, C.c_int, _f64p]
        L.oracle_deep_scores.restype = C.c_int
        L.oracle_maxpool.argtypes = [_f64p, C.c_int, C.c_int, _f64p]
        L.oracle_maxpool.restype = None
        L.oracle_topk.argtypes = [_f64p, C.c_int, C.c_int, _i32p]
        L.oracle_topk.restype = None
        L.oracle_deep_unit.argtypes = [_f64p, _f64p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double,
                                       C.c_int, C.c_int, C.c_int, _f64p, _i32p]
        L.oracle_deep_unit.restype = C.c_int
        L.oracle_magnitudes.argtypes = [_f64p, C.c_int, C.c_int, _f64p]
        L.oracle_magnitudes.restype = None
        L.oracle_cos.argtypes = [_f64p, _f64p, C.c_int, C.c_int, C.c_int]
        L.oracle_cos.restype = C.c_double
        L.oracle_adjacency.argtypes = [_f64p, _f64p, C.c_int, C.c_int, C.c_double, _u32p, _i32p]
        L.oracle_adjacency.restype = None
        L.oracle_adjacency_row.argtypes = [_f64p, _f64p, C.c_int, C.c_int, C.c_double, C.c_int, _u32p]
        L.oracle_adjacency_row.restype = None
        L.oracle_merge_literal.argtypes = [_u32p, C.c_int, _i32p, _i32p]
        L.oracle_merge_literal.restype = C.c_int
        L.oracle_merge_incremental.argtypes = [_u32p, C.c_int, _i32p, _i32p]
        L.oracle_merge_incremental.restype = C.c_int
        L.oracle_cap_assign.argtypes = [_f64p, _f64p, C.c_int, C.c_int, _i32p, C.c_int, C.c_int, _i32p]
        L.oracle_cap_assign.restype = C.c_int
        L.oracle_codebook.argtypes = [_f64p, _f64p, C.c_int, _i32p, C.c_int, _f64p]
        L.oracle_codebook.restype = None
        L.oracle_shallow_unit.argtypes = [_f64p, C.c_int, C.c_int, C.c_double, C.c_int, C.c_int,
                                          _f64p, _u32p, _i32p, _i32p, _i32p, _f64p]
        L.oracle_shallow_unit.restype = C.c_int
        L.oracle_reconstruct.argtypes = [_f64p, _i32p, _f64p, C.c_int, C.c_int, _f64p]
        L.oracle_reconstruct.restype = None
        L.oracle_decode_merge.argtypes = [_f64p, C.c_int, C.c_int, _f64p, C.c_int, C.c_double, C.c_int, C.c_int,
                                          _f64p, _i32p, _f64p, _i32p]
        L.oracle_decode_merge.restype = C.c_int
        L.oracle_layer_ratios.argtypes = [C.c_double, C.c_int, C.c_int, C.c_int, C.c_double, _f64p]
        L.oracle_layer_ratios.restype = None
        L.oracle_layer_budgets.argtypes = [C.c_double, C.c_int, C.c_int, C.c_int, C.c_double, _i32p]
        L.oracle_layer_budgets.restype = None
        L.oracle_reserve_ratio.argtypes = [C.c_double, C.c_double, C.c_double, C.c_int, C.c_int, C.c_int, C.c_int, _f64p]
        L.oracle_reserve_ratio.restype = None
        _lib = L
    return _lib


def _c(x, dt=np.float64):
    return np.ascontiguousarray(x, dtype=dt)


def words(n: int) -> int:
    return (n + 31) // 32


# ---------------------------------------------------------------- eviction path

def deep_scores(Q, K, scale, norm_mode=0):
    """Q [hn, lw, d], K [l, d] (float64) -> ac' [l - lw]."""
    Q, K = _c(Q), _c(K)
    hn, lw, d = Q.shape
    l = K.shape[0]
    out = np.zeros(max(l - lw, 0), dtype=np.float64)
    rc = lib().oracle_deep_scores(Q, K, hn, lw, l, d, float(scale), int(norm_mode), out)
    if rc:
        raise ValueError(f"oracle_deep_scores rc={rc}")
    return out


def maxpool(x, P):
    x = _c(x)
    out = np.empty_like(x)
    lib().oracle_maxpool(x, len(x), int(P), out)
    return out


def topk(p, k):
    p = _c(p)
    idx = np.empty(k, dtype=np.int32)
    lib().oracle_topk(p, len(p), int(k), idx)
    return idx


def deep_unit(Q, K, scale, P, budget, norm_mode=0):
    """One (batch, kv-head) eviction problem -> (pooled [l_c], kept [min(budget,l)])."""
    Q, K = _c(Q), _c(K)
    hn, lw, d = Q.shape
    l = K.shape[0]
    pooled = np.zeros(max(l - lw, 0), dtype=np.float64)
    kept = np.empty(min(budget, l), dtype=np.int32)
    rc = lib().oracle_deep_unit(Q, K, hn, lw, l, d, float(scale), int(norm_mode), int(P), int(budget),
                                pooled, kept)
    if rc < 0:
        raise ValueError(f"oracle_deep_unit rc={rc}")
    return pooled, kept[:rc]


def deep_layer(Q, K, group_size, scale, P, budget, norm_mode=0, threads=8):
    """Q [B, H*hn, lw, d], K [B, H, l, d] float64 -> pooled [B,H,l_c], kept [B,H,min(budget,l)]."""
    B, H, l, d = K.shape
    lw = Q.shape[2]
    units = [(b, h) for b in range(B) for h in range(H)]

    def run(u):
        b, h = u
        return deep_unit(Q[b, h * group_size:(h + 1) * group_size], K[b, h], scale, P, budget, norm_mode)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(run, units))
    pooled = np.stack([r[0] for r in res]).reshape(B, H, l - lw)
    kept = np.stack([r[1] for r in res]).reshape(B, H, -1)
    return pooled, kept


# ---------------------------------------------------------------- codebook path

def magnitudes(X):
    X = _c(X)
    m = np.empty(X.shape[0], dtype=np.float64)
    lib().oracle_magnitudes(X, X.shape[0], X.shape[1], m)
    return m


def cos(X, m, a, b):
    X = _c(X)
    return lib().oracle_cos(X, _c(m), X.shape[1], int(a), int(b))


def adjacency(X, theta, m=None):
    X = _c(X)
    n, d = X.shape
    if m is None:
        m = magnitudes(X)
    G = np.zeros((n, words(n)), dtype=np.uint32)
    deg = np.zeros(n, dtype=np.int32)
    lib().oracle_adjacency(X, _c(m), n, d, float(theta), G, deg)
    return G, deg


def adjacency_row(X, theta, a, m=None):
    X = _c(X)
    n, d = X.shape
    if m is None:
        m = magnitudes(X)
    row = np.zeros(words(n), dtype=np.uint32)
    lib().oracle_adjacency_row(X, _c(m), n, d, float(theta), int(a), row)
    return row


def merge(G, literal=False):
    """Bit-packed adjacency [n, words(n)] -> (picks [n_codes], ref [n])."""
    G = _c(G, np.uint32)
    n = G.shape[0]
    picks = np.full(max(n, 1), -1, dtype=np.int32)
    ref = np.full(max(n, 1), -1, dtype=np.int32)
    fn = lib().oracle_merge_literal if literal else lib().oracle_merge_incremental
    nc = fn(G, n, picks, ref)
    return picks[:nc].copy(), ref[:n].copy()


def shallow_unit(X, theta, cap, literal=False):
    """One (batch, kv-head, K|V) codebook problem.  X [n, d] float64.
    Returns dict(mag, G, deg, picks (uncapped pick order), n_codes_uncapped, n_codes, ref, C)."""
    X = _c(X)
    n, d = X.shape
    mag = np.empty(n, dtype=np.float64)
    G = np.zeros((n, words(n)), dtype=np.uint32)
    deg = np.zeros(n, dtype=np.int32)
    picks = np.full(max(n, 1), -1, dtype=np.int32)
    ref = np.full(max(n, 1), -1, dtype=np.int32)
    keep = min(cap, n)
    Cb = np.zeros((max(keep, 1), d), dtype=np.float64)
    nc = lib().oracle_shallow_unit(X, n, d, float(theta), int(cap), int(bool(literal)),
                                   mag, G, deg, picks, ref, Cb)
    k = min(nc, cap)
    return dict(mag=mag, G=G, deg=deg, picks=picks[:nc].copy(), n_codes_uncapped=nc, n_codes=k,
                ref=ref[:n].copy(), C=Cb[:k].copy())


def shallow_unit_caps(X, theta, caps):
    """One codebook problem under several caps: Eq. 8, Eq. 9 and the loop of Alg. 1 run once (they
    do not depend on the cap), then the cap step and the codebook rows per cap, by the same C
    functions oracle_shallow_unit calls in the same order.  Returns {cap: dict as shallow_unit,
    without G and deg}."""
    X = _c(X)
    n, d = X.shape
    mag = magnitudes(X)
    G, deg = adjacency(X, theta, mag)
    picks, ref0 = merge(G)
    del G
    nc = len(picks)
    out = {}
    for cap in caps:
        ref = ref0.copy()
        lib().oracle_cap_assign(X, mag, n, d, picks, nc, int(cap), ref)
        k = min(nc, int(cap))
        Cb = np.zeros((max(k, 1), d), dtype=np.float64)
        lib().oracle_codebook(X, mag, d, picks, k, Cb)
        out[int(cap)] = dict(mag=mag, picks=picks, n_codes_uncapped=nc, n_codes=k, ref=ref, C=Cb[:k].copy())
    return out


def shallow_layer(X, theta, cap, threads=8):
    """X [B, H, n, d] float64 -> list of per-unit dicts in (b, h) order."""
    B, H = X.shape[:2]
    units = [(b, h) for b in range(B) for h in range(H)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda u: shallow_unit(X[u[0], u[1]], theta, cap), units))


def decode_merge(X, Cb, theta, cap, literal=False):
    """Decode-time merge of the new tokens X [m, d] into the stored codebook Cb [nc, d] (float64
    values of the stored rows).  Returns dict(mag, ref, C_new (rows appended), n_found (entries
    needed in total), n_codes (entries stored afterwards), n_matched)."""
    X = _c(X)
    m, d = X.shape
    Cb = _c(Cb).reshape(-1, d)
    nc = Cb.shape[0]
    mag = np.empty(m, dtype=np.float64)
    ref = np.full(max(m, 1), -1, dtype=np.int32)
    C_new = np.zeros((max(m, 1), d), dtype=np.float64)
    nm = np.zeros(1, dtype=np.int32)
    Cin = Cb if nc else np.zeros((1, d), dtype=np.float64)
    found = lib().oracle_decode_merge(X, m, d, Cin, nc, float(theta), int(cap), int(bool(literal)),
                                      mag, ref, C_new, nm)
    stored = max(nc, min(found, cap))
    return dict(mag=mag, ref=ref[:m].copy(), C_new=C_new[:stored - nc].copy(), n_found=found,
                n_codes=stored, n_matched=int(nm[0]))


def reconstruct(Cb, ref, mag):
    Cb = _c(Cb)
    n, d = len(ref), Cb.shape[1]
    out = np.empty((n, d), dtype=np.float64)
    lib().oracle_reconstruct(Cb, _c(ref, np.int32), _c(mag), n, d, out)
    return out


def layer_ratios(r, l, lw, m, beta=0.05):
    out = np.empty(m, dtype=np.float64)
    lib().oracle_layer_ratios(float(r), int(l), int(lw), int(m), float(beta), out)
    return out


def layer_budgets(r, l, lw, m, beta=0.05):
    out = np.empty(m, dtype=np.int32)
    lib().oracle_layer_budgets(float(r), int(l), int(lw), int(m), float(beta), out)
    return out


def reserve_ratio(kept, total, entries, dh=128, int_bit=16, key_bit=16, mag_bit=None):
    out = np.empty(4, dtype=np.float64)
    lib().oracle_reserve_ratio(float(kept), float(total), float(entries), int(dh), int(int_bit), int(key_bit),
                               int(key_bit if mag_bit is None else mag_bit), out)
    return out
