"""Helpers for the GPU parity tests: run the HIP library on numpy inputs and compare with the oracle."""
import numpy as np
import torch

import oracle as O
import paper_2406_11257_amd as X

f32 = np.float32


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_compress(ctx, cases, alpha=5e-5, beta=2.0, nbits=4, iters=10, want_recon=True, blob_cap=None, flags=0):
    """cases: list of (Wp, W, m, v) numpy arrays.  Returns list of dicts (blob bytes, stats, W_recon)."""
    dev, keep = [], []
    for (Wp, W, m, v) in cases:
        n = W.size
        cap = X.excp_blob_bound(n, 32 if flags & 4 else nbits) if blob_cap is None else blob_cap
        blob = torch.zeros(cap + 64, dtype=torch.uint8, device="cuda")
        blob[cap:] = 0xAB                       # canary behind the capacity
        Wout = torch.full((n,), 7.0, dtype=torch.float32, device="cuda") if want_recon else None
        t = (to_dev(Wp), to_dev(W), to_dev(m), to_dev(v), blob[:cap], Wout)
        dev.append(t)
        keep.append((blob, cap))
    ctx.excp_compress_tensors(dev, alpha, beta, nbits, iters, flags)
    rc, stats = ctx.excp_collect(check=False)
    out = []
    for (t, (blob, cap), st) in zip(dev, keep, stats):
        full = blob.cpu().numpy()
        assert np.all(full[cap:] == 0xAB), "write past blob_cap"
        nb = int(st.blob_bytes)
        out.append(dict(blob=full[:nb].tobytes() if st.status == 0 else b"", stats=st, dev=t,
                        W_recon=None if t[5] is None else t[5].cpu().numpy(), blob_dev=blob[:cap]))
    return rc, out


def gpu_decompress(ctx, Wp, blob_bytes_np, n, want=(True, True, True)):
    blob = torch.from_numpy(np.frombuffer(blob_bytes_np, dtype=np.uint8).copy()).cuda()
    if blob.numel() % 16:
        blob = torch.cat([blob, torch.zeros(16 - blob.numel() % 16, dtype=torch.uint8, device="cuda")])
    Wp_d = to_dev(Wp)
    outs = [torch.full((n,), 9.0, dtype=torch.float32, device="cuda") if w else None for w in want]
    rc = ctx.excp_decompress_step(Wp_d, blob, len(blob_bytes_np), outs[0], outs[1], outs[2], check=False)
    return rc, [None if o is None else o.cpu().numpy() for o in outs]


def compare_with_oracle(case, got, alpha, beta, nbits, iters, centre_rtol=1e-5):
    """Element-by-element comparison of one compressed tensor with the oracle.  Returns the oracle result."""
    Wp, W, m, v = case
    n = W.size
    ref = O.compress_step(Wp, W, m, v, alpha, beta, nbits, iters)
    st = got["stats"]
    assert st.status == 0, st.status
    # thresholds, counts: bit exact
    assert (st.n, st.n_w, st.n_o) == (n, ref.n_w, ref.n_o)
    assert f32(st.median_abs_dw).tobytes() == f32(ref.median).tobytes()
    assert st.abs_sum_m == ref.abs_sum_m
    assert f32(st.mean_abs_m).tobytes() == f32(ref.mean_abs_m).tobytes()
    assert f32(st.t_w).tobytes() == f32(ref.t_w).tobytes()
    assert f32(st.r_o).tobytes() == f32(ref.r_o).tobytes()
    assert st.blob_bytes == len(ref.blob) == O.blob_size(n, ref.n_w, ref.n_o, nbits)
    g = O.parse_blob(got["blob"], n_expected=n)
    r = O.parse_blob(ref.blob)
    for key in ("nbits", "flags", "n", "n_w", "n_o", "iters", "blob_bytes"):
        assert g[key] == r[key], key
    for key in ("alpha", "beta", "median", "mean_abs_m", "t_w", "r_o"):
        assert g[key].tobytes() == r[key].tobytes(), key
    # masks: bit exact (including padding)
    assert np.array_equal(g["bitmap_w"], r["bitmap_w"])
    assert np.array_equal(g["bitmap_o"], r["bitmap_o"])
    # codebooks: entry 0 is +0, centres within tolerance
    K = (1 << nbits) - 1
    worst = 0.0
    for name, key in (("w", "book_w"), ("m", "book_m"), ("v", "book_v")):
        book = g[key]
        assert book[0] == 0 and not np.signbit(book[0])
        cg, co = book[1:].astype(np.float64), ref.C[name].astype(np.float64)
        assert np.all(np.diff(cg) >= 0)
        if ref.x[name].size:
            scale = np.abs(co).max()
            err = np.abs(cg - co) / np.maximum(np.abs(co), 1e-3 * scale)
            worst = max(worst, float(err.max()))
            assert err.max() <= centre_rtol, (name, err.max())
        else:
            assert not cg.any()
        # codes: given the GPU's own centres, the oracle's assignment must agree
        codes = O.unpack_codes(g["codes_" + name], ref.x[name].size, nbits)
        want = O.nearest_centre(ref.x[name], book[1:]) + 1
        mism = int((codes != want).sum())
        assert mism <= max(0, int(1e-6 * codes.size)), (name, mism)
        assert codes.size == 0 or (codes.min() >= 1 and codes.max() <= K)
    # objective agrees with what the oracle computes for the GPU's centres
    for name, val in (("w", st.obj_w), ("m", st.obj_m), ("v", st.obj_v)):
        x = ref.x[name]
        if x.size:
            a = O.nearest_centre(x, g["book_" + name][1:])
            o = O.objective(x, g["book_" + name][1:], a)
            assert abs(val - o) <= 1e-9 * max(o, 1e-300), (name, val, o)
        else:
            assert val == 0.0
    # whole blob identical when the centres are identical
    if all(np.array_equal(g[k], r[k]) for k in ("book_w", "book_m", "book_v")):
        assert got["blob"] == ref.blob
    # reconstruction kept for the next step: must equal Alg. 2 applied to the GPU's own blob
    if got["W_recon"] is not None:
        Wr, _, _ = O.decompress_step(Wp, got["blob"])
        assert np.array_equal(got["W_recon"].view(np.uint32), Wr.view(np.uint32))
    # compression ratio
    assert abs(12.0 * n / max(st.blob_bytes, 1) - ref.ratio) <= 1e-3 * ref.ratio
    return ref, worst
