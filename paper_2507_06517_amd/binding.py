"""Thin ctypes binding of the C ABI in ``include/spindle.h``.

Argument marshalling only: every step of both paths runs in the HIP kernels of
``libspindle.so``.  PyTorch supplies device memory and the current HIP stream.
The raw entry points keep their C names (``spindle_compress_deep`` ...); the
``compress_deep`` / ``compress_shallow`` / ``reconstruct`` helpers allocate the
outputs and the workspace and call them.  There is no fallback: a missing
library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libspindle.so")

F32, F16, BF16 = 0, 1, 2
NORM_PAPER, NORM_NONE = 0, 1
_DT = {"f32": F32, "f16": F16, "bf16": BF16}

# the first N_STATUS return a status code
EXPORTS = ["spindle_deep_workspace_bytes", "spindle_compress_deep", "spindle_shallow_workspace_bytes",
           "spindle_compress_shallow", "spindle_shallow_graph", "spindle_shallow_codebook",
           "spindle_shallow_layer_workspace_bytes", "spindle_compress_shallow_layer",
           "spindle_calibrate_mfma", "spindle_calibrate_similarity", "spindle_calibrate_copy",
           "spindle_shallow_stats", "spindle_reconstruct", "spindle_profile",
           "spindle_layer_budgets", "spindle_reserve_ratio", "spindle_decode_workspace_bytes", "spindle_decode_merge",
           "spindle_decode_merge_static",
           "spindle_profile_read", "spindle_decode_static_capacity",
           "spindle_last_error", "spindle_version"]
N_STATUS = 19


class KvDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_kv_heads", C.c_int32), ("group_size", C.c_int32),
                ("seq_len", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_t", C.c_int64)]


class SpindleError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"spindle status {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load libspindle.so (built by paper_2507_06517_amd.build); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2507_06517_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
        L.spindle_deep_workspace_bytes.argtypes = [C.POINTER(KvDesc), i32, C.POINTER(sz)]
        L.spindle_compress_deep.argtypes = [C.POINTER(KvDesc), vp, vp, vp, i32, i32, f32, i32, i32, vp, i32,
                                            vp, vp, vp, vp, vp, sz, vp]
        L.spindle_shallow_workspace_bytes.argtypes = [C.POINTER(KvDesc), i32, C.POINTER(sz)]
        for fn in (L.spindle_compress_shallow, L.spindle_shallow_graph, L.spindle_shallow_codebook):
            fn.argtypes = [C.POINTER(KvDesc), vp, vp, f32, f32, i32] + [vp] * 14 + [vp, sz, vp]
        L.spindle_shallow_layer_workspace_bytes.argtypes = [C.POINTER(KvDesc), i32, C.POINTER(sz)]
        L.spindle_compress_shallow_layer.argtypes = [C.POINTER(KvDesc), vp, vp, f32, f32, i32] + [vp] * 10 + [vp, sz, vp]
        L.spindle_calibrate_mfma.argtypes = [i32, i32, vp, C.POINTER(C.c_double)]
        L.spindle_calibrate_copy.argtypes = [vp, vp, sz, vp, C.POINTER(C.c_double)]
        L.spindle_calibrate_similarity.argtypes = [C.POINTER(KvDesc), i32, vp, sz, i32, vp, C.POINTER(C.c_double)]
        L.spindle_reconstruct.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]
        L.spindle_profile.argtypes = [i32]
        L.spindle_profile_read.argtypes = [C.c_char_p, C.POINTER(C.c_float), i32]
        L.spindle_profile_read.restype = C.c_int32
        L.spindle_shallow_stats.argtypes = [C.POINTER(KvDesc), i32, vp, vp, C.POINTER(C.c_int32)]
        L.spindle_layer_budgets.argtypes = [C.c_double, i32, i32, i32, C.c_double, C.POINTER(C.c_int32),
                                            C.POINTER(C.c_double)]
        L.spindle_reserve_ratio.argtypes = [C.c_int64, C.c_int64, C.c_int64, i32, i32, i32, i32, C.POINTER(C.c_double)]
        L.spindle_decode_workspace_bytes.argtypes = [C.POINTER(KvDesc), i32, C.POINTER(sz)]
        L.spindle_decode_merge.argtypes = [C.POINTER(KvDesc), vp, f32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.spindle_decode_merge_static.argtypes = [C.POINTER(KvDesc), vp, f32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.spindle_decode_static_capacity.argtypes = []
        L.spindle_decode_static_capacity.restype = sz
        for name in EXPORTS[:N_STATUS]:
            getattr(L, name).restype = C.c_int
        L.spindle_last_error.restype = C.c_char_p
        L.spindle_version.restype = C.c_uint32
        _lib = L
    return _lib


def _check(code):
    if code != 0:
        raise SpindleError(code, lib().spindle_last_error().decode())


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def torch_dtype(dtype: str):
    import torch
    return {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]


def to_device(bits: np.ndarray, dtype: str, device="cuda"):
    """numpy device representation (see workloads) -> torch tensor on the GPU."""
    import torch
    if dtype == "bf16":
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(bits).to(device)


def to_host_bits(t, dtype: str) -> np.ndarray:
    import torch
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def desc_of(K, group_size: int, dtype: str) -> KvDesc:
    """Descriptor of a [B, H, l, d] tensor; a view with another memory order (say a cache stored as
    [B, l, H, d]) is described by its strides, the head dimension has to be contiguous."""
    B, H, l, d = K.shape
    if K.is_contiguous():
        return KvDesc(B, H, group_size, l, d, _DT[dtype])
    if K.stride(3) != 1:
        raise ValueError("the head dimension of K and V must be contiguous")
    return KvDesc(B, H, group_size, l, d, _DT[dtype], K.stride(0), K.stride(1), K.stride(2))


# ------------------------------------------------------------------ raw calls (same names as the C ABI)

def spindle_deep_workspace_bytes(desc: KvDesc, window: int) -> int:
    out = C.c_size_t(0)
    _check(lib().spindle_deep_workspace_bytes(C.byref(desc), window, C.byref(out)))
    return out.value


def spindle_shallow_workspace_bytes(desc: KvDesc, n_tensors: int) -> int:
    out = C.c_size_t(0)
    _check(lib().spindle_shallow_workspace_bytes(C.byref(desc), n_tensors, C.byref(out)))
    return out.value


def spindle_compress_deep(desc, K, V, Qw, window, pool_kernel, scale, norm, budget, budgets, out_stride,
                          kept_idx, K_out, V_out, scores_out, workspace, workspace_bytes, stream=None):
    _check(lib().spindle_compress_deep(C.byref(desc), _ptr(K), _ptr(V), _ptr(Qw), window, pool_kernel,
                                       float(scale), norm, budget, _ptr(budgets), out_stride, _ptr(kept_idx),
                                       _ptr(K_out), _ptr(V_out), _ptr(scores_out), _ptr(workspace),
                                       workspace_bytes, stream if stream is not None else _stream()))


def _shallow_call(fn, desc, K, V, theta_k, theta_v, max_codes, Ck, Cv, n_codes_k, n_codes_v,
                  n_found_k, n_found_v, ref_k, ref_v, mag_k, mag_v, adj_k, adj_v, deg_k, deg_v,
                  workspace, workspace_bytes, stream=None):
    _check(fn(C.byref(desc), _ptr(K), _ptr(V), float(theta_k), float(theta_v),
              max_codes, _ptr(Ck), _ptr(Cv), _ptr(n_codes_k), _ptr(n_codes_v),
              _ptr(n_found_k), _ptr(n_found_v), _ptr(ref_k), _ptr(ref_v),
              _ptr(mag_k), _ptr(mag_v), _ptr(adj_k), _ptr(adj_v), _ptr(deg_k),
              _ptr(deg_v), _ptr(workspace), workspace_bytes,
              stream if stream is not None else _stream()))


def spindle_compress_shallow(*args, **kw):
    _shallow_call(lib().spindle_compress_shallow, *args, **kw)


def spindle_shallow_graph(*args, **kw):
    """First half of spindle_compress_shallow (same arguments): up to the neighbour lists."""
    _shallow_call(lib().spindle_shallow_graph, *args, **kw)


def spindle_shallow_codebook(*args, **kw):
    """Second half of spindle_compress_shallow (same arguments, same workspace)."""
    _shallow_call(lib().spindle_shallow_codebook, *args, **kw)


def spindle_shallow_stats(desc, n_tensors, workspace, stream=None):
    """-> int32 array [units * n_tensors, 16]: rounds, entries found, exact pairs, 0, phase us..."""
    n = desc.batch * desc.n_kv_heads * n_tensors
    buf = (C.c_int32 * (16 * n))()
    _check(lib().spindle_shallow_stats(C.byref(desc), n_tensors, _ptr(workspace),
                                       stream if stream is not None else _stream(), buf))
    return np.frombuffer(buf, dtype=np.int32).reshape(n, 16).copy()


def spindle_reconstruct(units, seq_len, head_dim, dtype, max_codes, Cb, ref, mag, out, stream=None):
    _check(lib().spindle_reconstruct(units, seq_len, head_dim, dtype, max_codes, _ptr(Cb), _ptr(ref),
                                     _ptr(mag), _ptr(out), stream if stream is not None else _stream()))


def spindle_layer_budgets(reserve_ratio, seq_len, window, n_layers, beta=0.05):
    """Returns (budgets int32 [n_layers], ratios float64 [n_layers])."""
    budgets = (C.c_int32 * n_layers)()
    ratios = (C.c_double * n_layers)()
    _check(lib().spindle_layer_budgets(float(reserve_ratio), int(seq_len), int(window), int(n_layers), float(beta),
                                       budgets, ratios))
    return np.array(budgets[:], dtype=np.int32), np.array(ratios[:], dtype=np.float64)


def spindle_reserve_ratio(kept_tokens, total_tokens, codebook_entries, head_dim=128, index_bits=16, elem_bits=16,
                          magnitude_bits=32):
    """Returns (r1, r2, r3, r) of one layer; the library's magnitudes are float32."""
    out = (C.c_double * 4)()
    _check(lib().spindle_reserve_ratio(int(kept_tokens), int(total_tokens), int(codebook_entries), int(head_dim),
                                       int(index_bits), int(elem_bits), int(magnitude_bits), out))
    return tuple(out[:])


def spindle_decode_workspace_bytes(desc: KvDesc, max_codes: int) -> int:
    out = C.c_size_t(0)
    _check(lib().spindle_decode_workspace_bytes(C.byref(desc), int(max_codes), C.byref(out)))
    return out.value


def spindle_decode_merge(desc, X_new, theta, max_codes, Cb, n_codes, n_found, n_matched, ref, mag, workspace,
                         workspace_bytes, stream=None):
    _check(lib().spindle_decode_merge(C.byref(desc), _ptr(X_new), float(theta), int(max_codes), _ptr(Cb),
                                      _ptr(n_codes), _ptr(n_found), _ptr(n_matched), _ptr(ref), _ptr(mag),
                                      _ptr(workspace), int(workspace_bytes), stream or _stream()))


def spindle_decode_merge_static(desc, X_new, theta, max_codes, Cb, n_codes, n_found, n_matched, ref, mag, stream=None):
    _check(lib().spindle_decode_merge_static(C.byref(desc), _ptr(X_new), float(theta), int(max_codes), _ptr(Cb),
                                             _ptr(n_codes), _ptr(n_found), _ptr(n_matched), _ptr(ref), _ptr(mag),
                                             stream or _stream()))


def spindle_decode_static_capacity() -> int:
    return int(lib().spindle_decode_static_capacity())


def decode_merge(X_new, dtype, theta, Cb, n_codes):
    """Merges X_new [B, H, m, d] into the codebooks Cb [B, H, cap, d] (updated in place, with n_codes
    [B, H] int32).  Returns dict(ref, mag, n_found, n_matched)."""
    import torch
    B, H, m, d = X_new.shape
    desc = KvDesc(B, H, 1, m, d, _DT[dtype])
    nbytes = spindle_decode_workspace_bytes(desc, Cb.shape[2])
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=X_new.device)
    out = dict(ref=torch.empty((B, H, m), dtype=torch.int32, device=X_new.device),
               mag=torch.empty((B, H, m), dtype=torch.float32, device=X_new.device),
               n_found=torch.empty((B, H), dtype=torch.int32, device=X_new.device),
               n_matched=torch.empty((B, H), dtype=torch.int32, device=X_new.device))
    spindle_decode_merge(desc, X_new, theta, Cb.shape[2], Cb, n_codes, out["n_found"], out["n_matched"],
                         out["ref"], out["mag"], ws, ws.numel())
    out["workspace"] = ws
    return out


def spindle_profile(mode) -> None:
    """0/False: off; 1/True: HIP events around every kernel; 2: around the similarity kernel only."""
    _check(lib().spindle_profile(int(mode)))


def spindle_profile_read(max_records: int = 4096):
    """-> list of (kernel name, milliseconds) in launch order; clears the records."""
    names = C.create_string_buffer(32 * max_records)
    ms = (C.c_float * max_records)()
    n = lib().spindle_profile_read(names, ms, max_records)
    if n < 0:
        raise SpindleError(4, "spindle_profile_read failed")
    return [(names.raw[i * 32:(i + 1) * 32].split(b"\0", 1)[0].decode(), float(ms[i])) for i in range(n)]


# ------------------------------------------------------------------ allocating helpers

@dataclass
class DeepPlan:
    """Pre-allocated outputs and workspace of one deep call shape."""
    desc: KvDesc
    window: int
    pool: int
    scale: float
    norm: int
    budget: int
    out_stride: int
    kept: object
    K_out: object
    V_out: object
    scores: object
    ws: object
    ws_bytes: int
    budgets: object = None

    def run(self, K, V, Qw):
        spindle_compress_deep(self.desc, K, V, Qw, self.window, self.pool, self.scale, self.norm, self.budget,
                              self.budgets, self.out_stride, self.kept, self.K_out, self.V_out, self.scores,
                              self.ws, self.ws_bytes)
        return self.kept, self.K_out, self.V_out, self.scores


def plan_deep(K, group_size, dtype, window, pool, budget, scale=None, norm=NORM_PAPER, want_scores=True,
              budgets=None, out_stride=None, with_v=True) -> DeepPlan:
    import torch
    B, H, l, d = K.shape
    desc = desc_of(K, group_size, dtype)
    if scale is None:
        scale = float(np.float32(1.0 / np.sqrt(d)))
    if out_stride is None:
        out_stride = min(budget, l)
    nbytes = spindle_deep_workspace_bytes(desc, window)
    dev = K.device
    return DeepPlan(desc, window, pool, scale, norm, budget, out_stride,
                    torch.empty((B, H, out_stride), dtype=torch.int32, device=dev),
                    torch.empty((B, H, out_stride, d), dtype=K.dtype, device=dev),
                    torch.empty((B, H, out_stride, d), dtype=K.dtype, device=dev) if with_v else None,
                    torch.empty((B, H, max(l - window, 1)), dtype=torch.float32, device=dev) if want_scores else None,
                    torch.empty(nbytes, dtype=torch.uint8, device=dev), nbytes, budgets)


def compress_deep(K, V, Qw, group_size, dtype, window, pool, budget, **kw):
    plan = plan_deep(K, group_size, dtype, window, pool, budget, with_v=V is not None, **kw)
    return plan.run(K, V, Qw)


@dataclass
class ShallowPlan:
    desc: KvDesc
    theta_k: float
    theta_v: float
    max_codes: int
    out: dict
    ws: object
    ws_bytes: int

    def _args(self, K, V):
        g = self.out.get
        return (self.desc, K, V, self.theta_k, self.theta_v, self.max_codes,
                g("C_k"), g("C_v"), g("n_codes_k"), g("n_codes_v"), g("n_found_k"), g("n_found_v"),
                g("ref_k"), g("ref_v"), g("mag_k"), g("mag_v"), g("adj_k"), g("adj_v"),
                g("deg_k"), g("deg_v"), self.ws, self.ws_bytes)

    def run(self, K, V):
        spindle_compress_shallow(*self._args(K, V))
        return self.out

    def run_graph(self, K, V):
        spindle_shallow_graph(*self._args(K, V))

    def run_codebook(self, K, V):
        spindle_shallow_codebook(*self._args(K, V))
        return self.out

    def stats(self):
        n_t = sum(1 for k in self.out if k.startswith("ref_"))
        return spindle_shallow_stats(self.desc, n_t, self.ws)


def plan_shallow(K, dtype, theta_k, theta_v, max_codes, tensors=("k", "v"), debug=False) -> ShallowPlan:
    import torch
    B, H, l, d = K.shape
    desc = desc_of(K, 1, dtype)
    nbytes = spindle_shallow_workspace_bytes(desc, len(tensors))
    dev = K.device
    out = {}
    for t in tensors:
        out[f"C_{t}"] = torch.empty((B, H, max_codes, d), dtype=K.dtype, device=dev)
        out[f"n_codes_{t}"] = torch.empty((B, H), dtype=torch.int32, device=dev)
        out[f"n_found_{t}"] = torch.empty((B, H), dtype=torch.int32, device=dev)
        out[f"ref_{t}"] = torch.empty((B, H, l), dtype=torch.int32, device=dev)
        out[f"mag_{t}"] = torch.empty((B, H, l), dtype=torch.float32, device=dev)
        if debug:
            out[f"adj_{t}"] = torch.empty((B, H, l, (l + 31) // 32), dtype=torch.int32, device=dev)
            out[f"deg_{t}"] = torch.empty((B, H, l), dtype=torch.int32, device=dev)
    return ShallowPlan(desc, theta_k, theta_v, max_codes, out,
                       torch.empty(nbytes, dtype=torch.uint8, device=dev), nbytes)


class OverlappedLayer:
    """Eviction and codebook calls of one layer on two streams.  The first half of the codebook call
    (similarity graph) fills the chip; during the second half (the loop of Alg. 1, one workgroup per
    problem for most of it) most compute units are idle, so the eviction call runs beside it on a
    side stream that waits for an event recorded between the halves.  Streams and events only:
    the calls and their arguments are those of the one-stream sequence."""

    def __init__(self, deep: "DeepPlan", shallow: "ShallowPlan"):
        import torch
        self.deep, self.shallow = deep, shallow
        self.side = torch.cuda.Stream()              # default priority
        self.fork, self.join = torch.cuda.Event(), torch.cuda.Event()

    def run(self, K, V, Qw):
        import torch
        main = torch.cuda.current_stream()
        self.shallow.run_graph(K, V)
        self.fork.record(main)
        # the second half is enqueued first: its chain of short dependent kernels is the longer of
        # the two and should not queue behind an eviction kernel
        out = self.shallow.run_codebook(K, V)
        self.side.wait_event(self.fork)
        with torch.cuda.stream(self.side):
            kept = self.deep.run(K, V, Qw)
            self.join.record(self.side)
        main.wait_event(self.join)                   # later work on the main stream sees both results
        return kept, out


class PipelinedLayers:
    """Consecutive layers (independent calls) in a software pipeline over `depth` sets of buffers, each
    with a main and a side stream.  Layer k+1's similarity phase starts when layer k's has ended, so it
    runs beside layer k's codebook phase and eviction call, which leave most of the chip idle; two
    similarity phases never share the chip.  Streams and events only: every layer is the same sequence
    of calls as in OverlappedLayer, and a set's buffers are reused only after all of its work is done."""

    def __init__(self, make_plans, depth=2):
        import torch
        self.sets = []
        for _ in range(depth):
            deep, shallow = make_plans()
            self.sets.append(dict(deep=deep, shallow=shallow, main=torch.cuda.Stream(), side=torch.cuda.Stream(),
                                  graph=torch.cuda.Event(), join=torch.cuda.Event(), done=torch.cuda.Event()))
        self.k = 0
        self.prev_graph = None
        self.ready = torch.cuda.Event()

    def run(self, K, V, Qw):
        """Enqueue one layer; returns its set (outputs in set['deep'] / set['shallow'].out, valid after finish())."""
        import torch
        s = self.sets[self.k % len(self.sets)]
        self.k += 1
        main, side = s["main"], s["side"]
        self.ready.record(torch.cuda.current_stream())       # the inputs are ready on the caller's stream
        main.wait_event(self.ready)
        if self.prev_graph is not None:
            main.wait_event(self.prev_graph)                 # one similarity phase at a time
        with torch.cuda.stream(main):
            s["shallow"].run_graph(K, V)
            s["graph"].record(main)
            s["shallow"].run_codebook(K, V)
        side.wait_event(s["graph"])
        with torch.cuda.stream(side):
            s["deep"].run(K, V, Qw)
            s["join"].record(side)
        main.wait_event(s["join"])                           # the set is free again once main gets here
        s["done"].record(main)
        self.prev_graph = s["graph"]
        return s

    def finish(self):
        """The caller's stream waits for every layer enqueued so far."""
        import torch
        cur = torch.cuda.current_stream()
        for s in self.sets:
            cur.wait_event(s["done"])


def compress_shallow(K, V, dtype, theta_k, theta_v, max_codes, debug=False):
    ref = K if K is not None else V
    tensors = tuple(t for t, x in (("k", K), ("v", V)) if x is not None)
    plan = plan_shallow(ref, dtype, theta_k, theta_v, max_codes, tensors, debug)
    return plan.run(K, V)


def spindle_shallow_layer_workspace_bytes(desc: KvDesc, n_tensors: int) -> int:
    out = C.c_size_t(0)
    _check(lib().spindle_shallow_layer_workspace_bytes(C.byref(desc), int(n_tensors), C.byref(out)))
    return out.value


def spindle_compress_shallow_layer(desc, K, V, theta_k, theta_v, max_codes, Ck, Cv, n_codes_k, n_codes_v, n_found_k,
                                   n_found_v, ref_k, ref_v, mag_k, mag_v, workspace, workspace_bytes, stream=None):
    _check(lib().spindle_compress_shallow_layer(C.byref(desc), _ptr(K), _ptr(V), float(theta_k), float(theta_v),
                                                int(max_codes), _ptr(Ck), _ptr(Cv), _ptr(n_codes_k), _ptr(n_codes_v),
                                                _ptr(n_found_k), _ptr(n_found_v), _ptr(ref_k), _ptr(ref_v),
                                                _ptr(mag_k), _ptr(mag_v), _ptr(workspace), int(workspace_bytes),
                                                stream or _stream()))


def compress_shallow_layer(K, V, dtype, theta_k, theta_v, max_codes):
    """One codebook per layer over the rows of all heads.  K, V [B, H, l, d] (either may be None) ->
    dict(C_k [B, max_codes, d], n_codes_k [B], n_found_k [B], ref_k [B, H, l], mag_k [B, H, l], ... _v)."""
    import torch
    X = K if K is not None else V
    B, H, l, d = X.shape
    desc = desc_of(X, 1, dtype)
    tensors = [t for t, x in (("k", K), ("v", V)) if x is not None]
    nbytes = spindle_shallow_layer_workspace_bytes(desc, len(tensors))
    dev = X.device
    out = {}
    for t in tensors:
        out[f"C_{t}"] = torch.empty((B, max_codes, d), dtype=X.dtype, device=dev)
        out[f"n_codes_{t}"] = torch.empty((B,), dtype=torch.int32, device=dev)
        out[f"n_found_{t}"] = torch.empty((B,), dtype=torch.int32, device=dev)
        out[f"ref_{t}"] = torch.empty((B, H, l), dtype=torch.int32, device=dev)
        out[f"mag_{t}"] = torch.empty((B, H, l), dtype=torch.float32, device=dev)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    g = out.get
    spindle_compress_shallow_layer(desc, K, V, theta_k, theta_v, max_codes, g("C_k"), g("C_v"), g("n_codes_k"),
                                   g("n_codes_v"), g("n_found_k"), g("n_found_v"), g("ref_k"), g("ref_v"),
                                   g("mag_k"), g("mag_v"), ws, nbytes)
    out["workspace"] = ws
    return out


def spindle_calibrate_mfma(iters: int = 4096, pattern: int = 0, stream=None) -> float:
    """TFLOP/s of a register-resident fp16 MFMA loop on the whole chip (measurement aid); pattern 1 =
    operands with the signs and magnitudes of the similarity kernel's."""
    out = C.c_double(0.0)
    _check(lib().spindle_calibrate_mfma(int(iters), int(pattern), stream or _stream(), C.byref(out)))
    return out.value


def spindle_calibrate_copy(src, dst, stream=None) -> float:
    """GB/s (read + written) of a plain copy of src into dst (same-size device tensors; measurement aid)."""
    out = C.c_double(0.0)
    _check(lib().spindle_calibrate_copy(_ptr(src), _ptr(dst), int(src.numel() * src.element_size()),
                                        stream or _stream(), C.byref(out)))
    return out.value


def spindle_calibrate_similarity(plan: "ShallowPlan", mode: int = 0, stream=None) -> float:
    """Milliseconds of the similarity kernel's loop without its packing, on the unit vectors the
    plan's last run left in its workspace (measurement aid); mode 1 also without the streaming
    loads, mode 2 matrix instructions only."""
    out = C.c_double(0.0)
    n_t = sum(1 for k in plan.out if k.startswith("ref_"))
    _check(lib().spindle_calibrate_similarity(C.byref(plan.desc), n_t, _ptr(plan.ws), int(plan.ws_bytes),
                                              int(mode), stream or _stream(), C.byref(out)))
    return out.value


def reconstruct(Cb, ref, mag, dtype):
    import torch
    B, H, cap, d = Cb.shape
    l = ref.shape[-1]
    out = torch.empty((B, H, l, d), dtype=Cb.dtype, device=Cb.device)
    spindle_reconstruct(B * H, l, d, _DT[dtype], cap, Cb, ref, mag, out)
    return out
