"""GPU parity of the stored layout of Sec. 4.2 (one code per element, two 4-bit codes per byte): the
export from a compressed tensor and Alg. 2 from that layout, byte for byte against the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2406_11257_amd as X
from gpu_util import gpu_compress, to_dev
from test_gpu_parity import case

pytestmark = pytest.mark.gpu
f32 = np.float32
CANARY = 0xC5


@pytest.fixture(scope="module")
def ctx():
    c = X.Context(4 << 20, 6 << 20)
    yield c
    c.close()


def code_buffer(nbytes):
    t = torch.full((nbytes + 32,), CANARY, dtype=torch.uint8, device="cuda")
    return t


def export(ctx, outs, nbits, want=(True, True, True, True)):
    """Export every compressed tensor of `outs`; returns per tensor (head, cw, cm, cv) as numpy (None if not asked)."""
    items, bufs = [], []
    for o in outs:
        n = int(o["stats"].n)
        db = X.excp_dense_bytes(n, nbits)
        hb = X.excp_head_bytes(nbits)
        b = [code_buffer(hb) if want[0] else None] + [code_buffer(db) if w else None for w in want[1:]]
        bufs.append((b, hb, db))
        items.append((o["blob_dev"], int(o["stats"].blob_bytes), n, *b))
    ctx.excp_export_dense(items)
    rc, stats = ctx.excp_collect(check=False)
    res = []
    for (b, hb, db) in bufs:
        r = []
        for t, size in zip(b, (hb, db, db, db)):
            if t is None:
                r.append(None)
                continue
            a = t.cpu().numpy()
            assert np.all(a[size:] == CANARY), "write past the end of a code tensor"
            r.append(a[:size].copy())
        res.append(r)
    return rc, stats, res, bufs


def dense_decode(ctx, Wps, bufs, ns, want=(True, True, True)):
    items, outs = [], []
    for Wp, (b, hb, db), n in zip(Wps, bufs, ns):
        o = [torch.full((n,), 3.0, dtype=torch.float32, device="cuda") if w else None for w in want]
        outs.append(o)
        items.append((to_dev(Wp), b[0], hb, n, b[1], b[2], b[3], *o))
    ctx.excp_decompress_dense(items)
    rc, stats = ctx.excp_collect(check=False)
    return rc, stats, [[None if t is None else t.cpu().numpy() for t in o] for o in outs]


@pytest.mark.parametrize("nbits", [2, 3, 4, 5, 8])
def test_export_and_reconstruction_match_the_oracle(ctx, nbits):
    sizes = [0, 1, 2, 3, 7, 63, 64, 65, 4095, 4096, 4097, 8191, 12289, 100001, (1 << 20) + 5]
    cases = [case(n, 100 + i) for i, n in enumerate(sizes)]
    rc, outs = gpu_compress(ctx, cases, 5e-5, 2.0, nbits, 3)
    assert rc == 0
    rc, stats, res, bufs = export(ctx, outs, nbits)
    assert rc == 0
    for c, o, st, (head, cw, cm, cv) in zip(cases, outs, stats, res):
        h_ref, w_ref, m_ref, v_ref = O.export_dense(o["blob"])
        assert st.status == 0 and (st.n, st.n_w, st.n_o) == (c[0].size, o["stats"].n_w, o["stats"].n_o)
        assert head.tobytes() == h_ref
        assert cw.tobytes() == w_ref.tobytes() and cm.tobytes() == m_ref.tobytes() and cv.tobytes() == v_ref.tobytes()
    rc, stats, dec = dense_decode(ctx, [c[0] for c in cases], bufs, sizes)
    assert rc == 0
    for c, o, st, (Wr, mr, vr), (head, cw, cm, cv) in zip(cases, outs, stats, dec, res):
        W_ref, m_ref, v_ref = O.decompress_dense(c[0], head.tobytes(), cw, cm, cv)
        assert st.status == 0 and (st.n_w, st.n_o) == (o["stats"].n_w, o["stats"].n_o)
        assert Wr.tobytes() == W_ref.tobytes() and mr.tobytes() == m_ref.tobytes() and vr.tobytes() == v_ref.tobytes()
        assert Wr.tobytes() == o["W_recon"].tobytes()          # what compress kept for the next step


def test_every_keep_fraction_from_none_to_all(ctx):
    n = 70001
    for alpha, beta in [(0.0, 0.0), (1e-5, 0.5), (2e-4, 3.0), (1.0, 2.0)]:
        cases = [case(n, 7)]
        rc, outs = gpu_compress(ctx, cases, alpha, beta, 4, 2)
        assert rc == 0
        rc, stats, res, bufs = export(ctx, outs, 4)
        assert rc == 0
        ref = O.export_dense(outs[0]["blob"])
        for got, want in zip(res[0][1:], ref[1:]):
            assert got.tobytes() == want.tobytes()
        rc, stats, dec = dense_decode(ctx, [cases[0][0]], bufs, [n])
        assert rc == 0 and dec[0][0].tobytes() == outs[0]["W_recon"].tobytes()


def test_outputs_are_optional(ctx):
    n = 50003
    cases = [case(n, 11)]
    rc, outs = gpu_compress(ctx, cases, 5e-5, 2.0, 4, 2)
    ref = O.export_dense(outs[0]["blob"])
    for want in [(False, True, False, False), (True, False, True, False), (False, False, False, True), (False, False, False, False)]:
        rc, stats, res, bufs = export(ctx, outs, 4, want)
        assert rc == 0 and stats[0].status == 0
        for got, r, w in zip(res[0], (np.frombuffer(ref[0], np.uint8),) + ref[1:], want):
            assert (got is None) == (not w)
            if w:
                assert got.tobytes() == r.tobytes()
    rc, stats, res, bufs = export(ctx, outs, 4)
    full = O.decompress_dense(cases[0][0], ref[0], *ref[1:])
    for want in [(True, False, False), (False, True, False), (False, False, True), (False, True, True)]:
        rc, stats, dec = dense_decode(ctx, [cases[0][0]], bufs, [n], want)
        assert rc == 0
        for got, r, w in zip(dec[0], full, want):
            assert (got is None) == (not w)
            if w:
                assert got.tobytes() == r.tobytes()


def test_minus_zero_survives_and_in_place_update(ctx):
    n = 9001
    Wp, W, m, v = case(n, 13)
    Wp[:100] = -0.0
    W[:100] = -0.0
    rc, outs = gpu_compress(ctx, [(Wp, W, m, v)], 5e-5, 2.0, 4, 2)
    rc, stats, res, bufs = export(ctx, outs, 4)
    b, hb, db = bufs[0]
    Wd = to_dev(Wp)
    ctx.excp_decompress_dense([(Wd, b[0], hb, n, b[1], None, None, Wd, None, None)])     # output over the input
    rc, _ = ctx.excp_collect(check=False)
    got = Wd.cpu().numpy()
    assert rc == 0 and got.tobytes() == outs[0]["W_recon"].tobytes() and np.all(np.signbit(got[:100]))


def test_many_tensors_across_groups(ctx):
    g = np.random.default_rng(5)
    sizes = [int(x) for x in g.integers(1, 300000, 60)] + [3 << 20, (3 << 20) + 1]
    cases = [case(n, 500 + i) for i, n in enumerate(sizes)]
    rc, outs = gpu_compress(ctx, cases, 5e-5, 2.0, 4, 1)
    assert rc == 0
    rc, stats, res, bufs = export(ctx, outs, 4)
    assert rc == 0
    for o, (head, cw, cm, cv) in zip(outs, res):
        ref = O.export_dense(o["blob"])
        assert head.tobytes() == ref[0] and cw.tobytes() == ref[1].tobytes()
        assert cm.tobytes() == ref[2].tobytes() and cv.tobytes() == ref[3].tobytes()
    rc, stats, dec = dense_decode(ctx, [c[0] for c in cases], bufs, sizes)
    assert rc == 0
    for o, d in zip(outs, dec):
        assert d[0].tobytes() == o["W_recon"].tobytes()


def test_damage_and_argument_errors(ctx):
    n = 5001                                                         # odd: the last byte has an unused half
    cases = [case(n, 17), case(n, 18)]
    rc, outs = gpu_compress(ctx, cases, 5e-5, 2.0, 3, 2)
    rc, stats, res, bufs = export(ctx, outs, 3)
    assert rc == 0
    Wps = [c[0] for c in cases]
    # a code beyond the 3-bit codebook in the first tensor only
    bufs[0][0][1][100] = 0x0F
    rc, stats, dec = dense_decode(ctx, Wps, bufs, [n, n])
    assert rc == X.EXCP_E_BLOB and stats[0].status == X.EXCP_E_BLOB and stats[1].status == 0
    assert dec[1][0].tobytes() == outs[1]["W_recon"].tobytes()
    bufs[0][0][1][100] = 0
    # the unused half of the last byte
    last = X.excp_dense_bytes(n, 3) - 1
    keep = int(bufs[1][0][2][last])
    bufs[1][0][2][last] = keep | 0x10
    rc, stats, dec = dense_decode(ctx, Wps, bufs, [n, n])
    assert rc == X.EXCP_E_BLOB and stats[1].status == X.EXCP_E_BLOB
    bufs[1][0][2][last] = keep
    # header damage, short header, wrong n
    bufs[0][0][0][0] = 0x00
    rc, stats, dec = dense_decode(ctx, Wps, bufs, [n, n])
    assert rc == X.EXCP_E_BLOB and stats[0].status == X.EXCP_E_BLOB and stats[1].status == 0
    bufs[0][0][0][0] = 0x45
    rc, stats, dec = dense_decode(ctx, Wps, [(bufs[0][0], 100, bufs[0][2]), bufs[1]], [n, n])
    assert rc == X.EXCP_E_BLOB and stats[0].status == X.EXCP_E_BLOB
    rc, stats, dec = dense_decode(ctx, Wps, bufs, [n, n])
    assert rc == 0
    # export of a damaged blob
    bad = outs[0]["blob_dev"].clone()
    bad[0] = 0
    ctx.excp_export_dense([(bad, int(outs[0]["stats"].blob_bytes), n, None, bufs[0][0][1], None, None)])
    rc, stats = ctx.excp_collect(check=False)
    assert rc == X.EXCP_E_BLOB
    # argument errors: misaligned code tensor, missing input for a requested output
    b, hb, db = bufs[0]
    with pytest.raises(X.ExcpError):
        ctx.excp_export_dense([(outs[0]["blob_dev"], int(outs[0]["stats"].blob_bytes), n, None, b[1][1:], None, None)])
    Wout = torch.zeros(n, dtype=torch.float32, device="cuda")
    with pytest.raises(X.ExcpError):
        ctx.excp_decompress_dense([(to_dev(Wps[0]), b[0], hb, n, None, None, None, Wout, None, None)])
    with pytest.raises(X.ExcpError):
        ctx.excp_decompress_dense([(to_dev(Wps[0]), b[0], hb, n, b[1], None, None, None, Wout, None)])


@pytest.mark.parametrize("layout", ["dense", "blob"])
def test_archive_round_trip_through_the_gpu(ctx, layout):
    from paper_2406_11257_amd import archive as A
    sizes = [0, 5, 4097, 250001]
    cases = [case(n, 900 + i) for i, n in enumerate(sizes)]
    rc, outs = gpu_compress(ctx, cases, 5e-5, 2.0, 4, 3)
    assert rc == 0
    named = [(f"t{i}", o["blob_dev"], int(o["stats"].blob_bytes), n) for i, (o, n) in enumerate(zip(outs, sizes))]
    data = A.save_checkpoint(ctx, named, 4, layout=layout, preset=6, threads=4)
    assert len(data) < 12 * sum(sizes) / 8                  # far below the fp32 state it stands for
    back = A.load_checkpoint(ctx, data, {f"t{i}": to_dev(c[0]) for i, c in enumerate(cases)}, threads=4)
    for i, (c, o) in enumerate(zip(cases, outs)):
        W, m, v = back[f"t{i}"]
        ref = O.decompress_step(c[0], o["blob"])
        assert W.cpu().numpy().tobytes() == ref[0].tobytes() == o["W_recon"].tobytes()
        assert m.cpu().numpy().tobytes() == ref[1].tobytes() and v.cpu().numpy().tobytes() == ref[2].tobytes()


def test_prepared_batches_of_the_other_calls(ctx):
    # export, reconstruction from the stored layout and Alg. 3 from argument arrays marshalled once
    cases = [case(150001, 911), case(4097, 912)]
    rc, outs = gpu_compress(ctx, cases, iters=3)
    assert rc == 0
    items, bufs = [], []
    for o in outs:
        n = int(o["stats"].n)
        b = [code_buffer(X.excp_head_bytes(4))] + [code_buffer(X.excp_dense_bytes(n, 4)) for _ in range(3)]
        bufs.append(b)
        items.append((o["blob_dev"], int(o["stats"].blob_bytes), n, *b))
    exp = ctx.prepare_export_dense(items)
    assert isinstance(exp, X.PreparedBatch) and exp.kind == "export_dense"
    dec_items, dec_outs = [], []
    for c, o, b in zip(cases, outs, bufs):
        n = c[0].size
        res = [torch.zeros(n, device="cuda") for _ in range(3)]
        dec_outs.append(res)
        dec_items.append((to_dev(c[0]), b[0], X.excp_head_bytes(4), n, b[1], b[2], b[3], *res))
    dec = ctx.prepare_decompress_dense(dec_items)
    chains = ctx.prepare_chain([(to_dev(c[0]), [o["blob_dev"]], [int(o["stats"].blob_bytes)],
                                 torch.zeros(c[0].size, device="cuda"), None, None) for c, o in zip(cases, outs)])
    for rep in range(2):
        for b in bufs:
            for t in b:
                t.fill_(CANARY)
        ctx.excp_export_dense(exp)
        ctx.excp_collect()
        ctx.excp_decompress_dense(dec)
        ctx.excp_collect()
        ctx.excp_reconstruct_chain(chains)
        ctx.excp_collect()
        for c, o, b, res, ch in zip(cases, outs, bufs, dec_outs, chains.keep[0]):
            n = c[0].size
            ref = O.export_dense(o["blob"])
            for got, want in zip(b[1:], ref[1:]):
                assert got[:X.excp_dense_bytes(n, 4)].cpu().numpy().tobytes() == want.tobytes(), rep
            W2, m2, v2 = O.decompress_step(c[0], o["blob"])
            assert res[0].cpu().numpy().tobytes() == W2.tobytes() and res[1].cpu().numpy().tobytes() == m2.tobytes()
            assert res[2].cpu().numpy().tobytes() == v2.tobytes()
            assert ch[3].cpu().numpy().tobytes() == W2.tobytes()
    with pytest.raises(TypeError):
        ctx.excp_export_dense(dec)
