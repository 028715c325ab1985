"""GPU parity of the remaining modes of the paper's ablation tables: prune without quantisation
(Table "abl"), no residual, no pruning, and the moment mask without the weights-to-momentum check
(Table "vit").  Blob for blob and element for element against the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2406_11257_amd as X
from gpu_util import gpu_compress, gpu_decompress, to_dev
from test_gpu_parity import case

pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def ctx():
    c = X.Context(4 << 20, 6 << 20)
    yield c
    c.close()


def check_mode(ctx, cases, alpha, beta, nbits, iters, flags):
    rc, outs = gpu_compress(ctx, cases, alpha, beta, nbits, iters, flags=flags)
    assert rc == 0
    refs = []
    for c, o in zip(cases, outs):
        ref = O.compress_step(*c, alpha, beta, nbits, iters, flags=flags)
        st = o["stats"]
        assert st.status == 0 and (st.n, st.n_w, st.n_o) == (c[0].size, ref.n_w, ref.n_o)
        assert st.blob_bytes == len(ref.blob)
        assert o["blob"] == ref.blob
        assert o["W_recon"].tobytes() == ref.W_recon.tobytes()
        rc2, dec = gpu_decompress(ctx, c[0], o["blob"], c[0].size)
        assert rc2 == 0
        assert dec[0].tobytes() == ref.W_recon.tobytes() and dec[1].tobytes() == ref.m_recon.tobytes()
        assert dec[2].tobytes() == ref.v_recon.tobytes()
        refs.append(ref)
    return outs, refs


SIZES = [0, 1, 2, 5, 63, 64, 65, 2047, 2049, 4095, 4097, 8193, 70001, (1 << 20) + 3]


@pytest.mark.parametrize("flags", [4, 5, 6])
def test_prune_only_mode(ctx, flags):
    cases = [case(n, 300 + i) for i, n in enumerate(SIZES)]
    alpha = 0.7 if flags & 2 else 5e-5
    outs, refs = check_mode(ctx, cases, alpha, 2.0, 4, 10, flags)
    for c, o, r in zip(cases, outs, refs):
        assert o["stats"].blob_bytes == X.excp_blob_size(c[0].size, r.n_w, r.n_o, 32)
        assert o["stats"].obj_w == 0.0 and o["stats"].obj_m == 0.0


@pytest.mark.parametrize("alpha,beta", [(0.0, 0.0), (2e-4, 3.0), (1.0, 2.0)])
def test_prune_only_from_everything_kept_to_nothing_kept(ctx, alpha, beta):
    cases = [case(n, 340 + i) for i, n in enumerate([5, 4097, 300001])]
    check_mode(ctx, cases, alpha, beta, 4, 0, 4)


def test_prune_only_blobs_in_mixed_batches_and_where_they_are_refused(ctx):
    n = 50001
    cases = [case(n, 360), case(n, 361), case(n, 362)]
    rc, raw = gpu_compress(ctx, cases[:2], flags=4)
    rc, coded = gpu_compress(ctx, cases[2:], flags=0)
    assert rc == 0
    both = [raw[0], coded[0], raw[1]]
    Wout = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in both]
    mout = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in both]
    vout = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in both]
    order = [cases[0], cases[2], cases[1]]
    ctx.excp_decompress_tensors([(to_dev(c[0]), o["blob_dev"], int(o["stats"].blob_bytes), n, W, m, v)
                                 for c, o, W, m, v in zip(order, both, Wout, mout, vout)])
    rc, stats = ctx.excp_collect(check=False)
    assert rc == 0
    for c, o, W, m, v in zip(order, both, Wout, mout, vout):
        ref = O.decompress_step(c[0], o["blob"])
        assert W.cpu().numpy().tobytes() == ref[0].tobytes() and m.cpu().numpy().tobytes() == ref[1].tobytes()
        assert v.cpu().numpy().tobytes() == ref[2].tobytes()
    # no chain reconstruction and no export of code tensors from a blob without codes
    o = raw[0]
    ctx.excp_reconstruct_chain([(to_dev(cases[0][0]), [o["blob_dev"]], [int(o["stats"].blob_bytes)], Wout[0], None, None)])
    rc, stats = ctx.excp_collect(check=False)
    assert rc == X.EXCP_E_BLOB
    codes = torch.zeros(X.excp_dense_bytes(n, 4) + 16, dtype=torch.uint8, device="cuda")
    ctx.excp_export_dense([(o["blob_dev"], int(o["stats"].blob_bytes), n, None, codes, None, None)])
    rc, stats = ctx.excp_collect(check=False)
    assert rc == X.EXCP_E_BLOB
    # capacity: the bound for 4-bit codes is too small for fp32 values when many survive
    with_cap = X.excp_blob_bound(n, 4)
    rc, out = gpu_compress(ctx, [cases[0]], 0.0, 0.0, 4, 0, flags=4, blob_cap=with_cap)
    assert rc == X.EXCP_E_CAP and out[0]["stats"].status == X.EXCP_E_CAP
    # damage: the flag without the width, and the width without the flag
    good = bytearray(raw[0]["blob"])
    for off, val in ((12, 0), (8, 4)):
        b = bytearray(good); b[off] = val
        rc, _ = gpu_decompress(ctx, cases[0][0], bytes(b), n)
        assert rc == X.EXCP_E_BLOB


def test_no_residual_and_no_pruning_need_no_switch(ctx):
    # Table "abl": without the residual the previous weights are zeros; without pruning alpha = beta = 0
    n = 200003
    Wp, W, m, v = case(n, 370)
    zeros = np.zeros(n, f32)
    outs, refs = check_mode(ctx, [(zeros, W, m, v)], 5e-5, 2.0, 4, 5, 0)
    assert refs[0].median == np.sort(np.abs(W))[(n - 1) // 2]            # the "residual" is the weight itself
    outs, refs = check_mode(ctx, [(Wp, W, m, v)], 0.0, 0.0, 4, 5, 0)
    assert refs[0].n_w == np.count_nonzero(W - Wp) and refs[0].n_o == np.count_nonzero((W - Wp != 0) & (m != 0))


@pytest.mark.parametrize("flags", [8, 9, 10, 12, 15])
def test_moment_mask_without_the_weights_to_momentum_check(ctx, flags):
    cases = [case(n, 400 + i) for i, n in enumerate(SIZES)]
    alpha = 0.7 if flags & 2 else 5e-5
    outs, refs = check_mode(ctx, cases, alpha, 1.0, 4, 3, flags)
    for c, o, r in zip(cases, outs, refs):
        assert o["stats"].blob_bytes == X.excp_blob_size_ex(c[0].size, r.n_w, r.n_o, 32 if flags & 4 else 4, flags)
    big = refs[-1]
    assert np.any(big.Mo & ~big.Mw) and big.n_o > 0


@pytest.mark.parametrize("alpha,beta,nbits", [(1.0, 0.0, 2), (0.0, 3.0, 8), (2e-4, 0.5, 5), (1.0, 0.5, 3)])
def test_no_w2m_from_no_weights_kept_to_all_moments_kept(ctx, alpha, beta, nbits):
    # alpha = 1 prunes (nearly) every weight while the moments stay: n_o far above n_w
    cases = [case(n, 440 + i) for i, n in enumerate([7, 4097, 262145])]
    outs, refs = check_mode(ctx, cases, alpha, beta, nbits, 2, 8)
    if alpha == 1.0:
        assert refs[-1].n_o > refs[-1].n_w


def test_no_w2m_through_the_stored_layout_and_the_chain(ctx):
    from test_gpu_dense import export, dense_decode
    n = 150001
    cases = [case(n, 460), case(4097, 461)]
    rc, outs = gpu_compress(ctx, cases, 5e-5, 1.0, 4, 2, flags=8)
    assert rc == 0
    rc, stats, res, bufs = export(ctx, outs, 4)
    assert rc == 0
    for o, (head, cw, cm, cv) in zip(outs, res):
        ref = O.export_dense(o["blob"])
        assert head.tobytes() == ref[0] and cw.tobytes() == ref[1].tobytes()
        assert cm.tobytes() == ref[2].tobytes() and cv.tobytes() == ref[3].tobytes()
    rc, stats, dec = dense_decode(ctx, [c[0] for c in cases], bufs, [n, 4097])
    assert rc == 0
    for c, o, d in zip(cases, outs, dec):
        ref = O.decompress_step(c[0], o["blob"])
        assert d[0].tobytes() == ref[0].tobytes() and d[1].tobytes() == ref[1].tobytes() and d[2].tobytes() == ref[2].tobytes()
    # a chain of two such checkpoints: the moments are those of the last one
    Wp, W, m, v = cases[0]
    r1 = O.compress_step(Wp, W, m, v, 5e-5, 1.0, 4, 2, flags=8)
    W2 = (W + np.random.default_rng(1).laplace(0, 1e-4, n).astype(f32)).astype(f32)
    rc, out2 = gpu_compress(ctx, [(r1.W_recon, W2, m, v)], 5e-5, 1.0, 4, 2, flags=8)
    Wout, mout, vout = (torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(3))
    ctx.excp_reconstruct_chain([(to_dev(Wp), [outs[0]["blob_dev"], out2[0]["blob_dev"]],
                                 [int(outs[0]["stats"].blob_bytes), int(out2[0]["stats"].blob_bytes)], Wout, mout, vout)])
    rc, stats = ctx.excp_collect(check=False)
    assert rc == 0
    ref = O.reconstruct_chain(Wp, [outs[0]["blob"], out2[0]["blob"]])
    assert Wout.cpu().numpy().tobytes() == ref[0].tobytes() and mout.cpu().numpy().tobytes() == ref[1].tobytes()
    assert vout.cpu().numpy().tobytes() == ref[2].tobytes()
    # damage: a count that only the other layout allows, and a flipped moment bit
    good = bytearray(outs[0]["blob"])
    b = bytearray(good); b[12] = 0                         # same bytes read as the default layout: sizes disagree
    rc, _ = gpu_decompress(ctx, Wp, bytes(b), n)
    assert rc == X.EXCP_E_BLOB
    p = O.parse_blob(bytes(good))
    off_bo = 80 + 12 * 16 + (8 * ((n + 63) // 64) + 15) // 16 * 16
    b = bytearray(good); b[off_bo + 5] ^= 0x04
    rc, _ = gpu_decompress(ctx, Wp, bytes(b), n)
    assert rc == X.EXCP_E_BLOB
    with pytest.raises(X.ExcpError):
        ctx.excp_compress_tensors([], 5e-5, 2.0, 4, 2, 64)
