"""spindle_decode_merge_static (the entry point that allocates nothing: its scratch memory is an
array inside the library) against spindle_decode_merge on the same inputs: every output must be
bit-identical, on two calls in a row that share the array, the second smaller than the first, so
that whatever the first call left in the array lies beside and behind what the second one uses.
The first call is also compared with the oracle."""
import numpy as np
import pytest

from paper_2507_06517_amd import workloads as wl

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]


def both_ways(sb, new, Cb, nc, dtype, theta):
    """Runs the workspace call and the static call on copies of the same inputs; returns both
    results as host arrays."""
    import torch
    B, H, m, d = new.shape
    cap = Cb.shape[2]
    desc = sb.KvDesc(B, H, 1, m, d, {"f32": sb.F32, "f16": sb.F16, "bf16": sb.BF16}[dtype])
    res = []
    for static in (False, True):
        X = sb.to_device(new, dtype)
        Cd, nd = sb.to_device(Cb, dtype), torch.from_numpy(nc.copy()).cuda()
        out = dict(ref=torch.full((B, H, m), -7, dtype=torch.int32, device="cuda"),
                   mag=torch.full((B, H, m), -1.0, dtype=torch.float32, device="cuda"),
                   n_found=torch.full((B, H), -7, dtype=torch.int32, device="cuda"),
                   n_matched=torch.full((B, H), -7, dtype=torch.int32, device="cuda"))
        if static:
            sb.spindle_decode_merge_static(desc, X, theta, cap, Cd, nd, out["n_found"], out["n_matched"],
                                           out["ref"], out["mag"])
        else:
            nbytes = sb.spindle_decode_workspace_bytes(desc, cap)
            assert nbytes <= sb.spindle_decode_static_capacity()
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            sb.spindle_decode_merge(desc, X, theta, cap, Cd, nd, out["n_found"], out["n_matched"], out["ref"],
                                    out["mag"], ws, nbytes)
        torch.cuda.synchronize()
        r = {k: v.cpu().numpy() for k, v in out.items()}
        r["C"] = sb.to_host_bits(Cd, dtype)
        r["n_codes"] = nd.cpu().numpy()
        res.append(r)
    return res


def test_static_entry_point_matches_the_workspace_one(oracle):
    from paper_2507_06517_amd import binding as sb
    from test_gpu_decode import stored_codebooks
    dtype, theta = "f16", float(np.float32(0.98))
    # first call: 3 problems x 300 new tokens against ~400 entries in a table of 1200 rows (three
    # slices of entries, 19 tiles of tokens); second: 2 problems x 37 tokens, a table of 500 rows
    for seed, H, m, cap in ((11, 3, 300, 1200), (12, 2, 37, 500)):
        pre, new = wl.decode_case(seed, dtype, B=1, H=H, n_prefill=600, m=m, novel_frac=0.3, novel_centroids=9)
        Cb, nc = stored_codebooks(oracle, pre, dtype, theta, cap, [[cap] * H])
        ws_res, st_res = both_ways(sb, new, Cb, nc, dtype, theta)
        for k in ws_res:
            assert np.array_equal(ws_res[k], st_res[k]), f"{k} differs between the two entry points (m = {m})"
        assert (st_res["n_matched"] > 0).all() and (st_res["n_found"] > nc).any()
        for h in range(H):
            k0 = int(nc[0, h])
            o = oracle.decode_merge(wl.to_f64(new[0, h], dtype), wl.to_f64(Cb[0, h, :k0], dtype), theta, cap)
            assert np.array_equal(st_res["ref"][0, h], o["ref"])
            assert np.array_equal(st_res["mag"][0, h], o["mag"].astype(np.float32))
            assert st_res["n_found"][0, h] == o["n_found"] and st_res["n_codes"][0, h] == o["n_codes"]
            assert st_res["n_matched"][0, h] == o["n_matched"]


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    from paper_2507_06517_amd import binding as sb
    B, H, m, cap = 4, 8, 1024, 4096             # 32 problems x 1024 tokens: 32 MiB of doubles alone
    desc = sb.KvDesc(B, H, 1, m, 128, sb.F16)
    assert sb.spindle_decode_workspace_bytes(desc, cap) > sb.spindle_decode_static_capacity()
    X = torch.zeros((B, H, m, 128), dtype=torch.float16, device="cuda")
    Cd = torch.zeros((B, H, cap, 128), dtype=torch.float16, device="cuda")
    nd = torch.zeros((B, H), dtype=torch.int32, device="cuda")
    ref = torch.full((B, H, m), -7, dtype=torch.int32, device="cuda")
    mag = torch.zeros((B, H, m), dtype=torch.float32, device="cuda")
    with pytest.raises(sb.SpindleError) as e:
        sb.spindle_decode_merge_static(desc, X, 0.98, cap, Cd, nd, nd.clone(), None, ref, mag)
    assert e.value.code == 2 and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (ref == -7).all()                    # nothing ran
