"""A seeded random campaign on the GPU against the oracle: every batch draws a code width, an
iteration count, thresholds, a combination of the switches (16-bit weight storage included) and eight
tensors of random sizes and structures (Laplace steps, a handful of distinct values, magnitudes spread
over eight decades, mostly-still weights, one-sided steps, constant steps, heavy tails).  Everything
the library produces is compared with the oracle bit for bit: counts, the blob, the reconstructed
weights, Alg. 2 from the blob, and the stored layout of Sec. 4.2."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2406_11257_amd as X
from test_gpu_w16 import bits, w_to_dev, w_to_host

pytestmark = pytest.mark.gpu
f32 = np.float32
EDGE_SIZES = [1, 2, 63, 64, 65, 2047, 2048, 2049, 4095, 4096, 4097, 8191, 8192, 8193]


@pytest.fixture(scope="module")
def ctx():
    c = X.Context(1 << 21, 4 << 20)
    yield c
    c.close()


@pytest.fixture(scope="module")
def ctx_wide():
    """The same limits, with the size thresholds of the library lowered so that every batch runs the
    kernel forms that otherwise only tensors of 2^28 elements (per-bucket totals and initial centres with
    sixteen waves, one workgroup per bucket) or 2^27 elements (several median-candidate lists) reach."""
    c = X.Context(1 << 21, 4 << 20)
    c.excp_set_param(X.EXCP_PARAM_WIDE_ELEMS, 1)
    c.excp_set_param(X.EXCP_PARAM_CAND_LIST_ELEMS, 65536)
    yield c
    c.close()


def draw_batch(seed, big=None):
    """big: None, or the weight-storage flags of a batch whose first two tensors are large (0.6 to 1.5 M
    elements), one of Laplace steps and one of a handful of distinct values."""
    g = np.random.default_rng(7700 + seed)
    nbits = int(g.integers(2, 9))
    iters = int(g.integers(0, 6))
    flags = int(g.integers(0, 16)) | int(g.choice([0, 0, 16, 32]))
    if big is not None:
        flags = (flags & 0xA) | big              # quantised, median of the residual, the storage asked for
        iters = max(iters, 2)
    alpha = float(g.choice([0.0, 1e-6, 5e-5, 1e-3, 1.0])) if g.random() < 0.5 else float(10 ** g.uniform(-7, 0))
    if flags & O.FLAG_NO_M2W:                      # a plain scalar threshold: of the order of the median itself
        alpha = float(g.choice([0.0, 0.3, 0.7, 1.5, 20.0]))
    beta = float(g.choice([0.0, 0.5, 2.0, 10.0]))
    if big is not None:                            # thresholds that keep a good share of every stream
        alpha, beta = (0.3 if flags & O.FLAG_NO_M2W else 5e-5), 0.5
    cases = []
    for q in range(8):
        n = int(g.choice(EDGE_SIZES)) if g.random() < 0.4 else int(g.integers(1, 90000))
        if g.random() < 0.15:
            n = int(g.integers(100000, 1500000))
        kind = int(g.integers(0, 7))
        if big is not None and q < 2:
            n, kind = int(g.integers(600000, 1500000)), q
        Wp = (g.standard_normal(n) * 0.02).astype(f32)
        if kind == 0:
            d = g.laplace(0, 1e-4, n)
        elif kind == 1:
            d = g.choice(np.array([-3e-4, -1e-4, 0.0, 1e-4, 2e-4, 5e-4]), n)
        elif kind == 2:
            d = g.standard_normal(n) * 10.0 ** g.uniform(-8, 0, n)
        elif kind == 3:
            d = np.where(g.random(n) < 0.2, g.laplace(0, 1e-4, n), 0.0)
        elif kind == 4:
            d = np.abs(g.laplace(0, 1e-4, n))
        elif kind == 5:
            d = np.full(n, 1e-4)
        else:
            d = g.standard_t(2, n) * 1e-4
        W = np.clip((Wp + d.astype(f32)).astype(f32), -6e4, 6e4)       # stays finite in fp16
        m = (g.standard_normal(n) * 5e-5).astype(f32)
        if kind in (1, 5):
            m = np.round(m * 2e5).astype(f32) / f32(2e5)               # tied moments
        if kind == 3:
            m[g.random(n) < 0.5] = 0
        v = (m.astype(np.float64) ** 2 * g.lognormal(0, 1, n) + 1e-16).astype(f32)
        if kind == 2:
            v[g.random(n) < 0.1] = 0
        cases.append((O.narrow(Wp, flags), O.narrow(W, flags), m, v))
    return nbits, iters, flags, alpha, beta, cases


@pytest.mark.parametrize("seed", range(24))
def test_random_batch(ctx, seed):
    run_batch(ctx, seed, None)


@pytest.mark.parametrize("seed", range(100, 110))
def test_random_batch_in_the_forms_for_very_large_tensors(ctx_wide, seed):
    run_batch(ctx_wide, seed, None)


@pytest.mark.parametrize("seed,storage", [(200, 0), (201, 16), (202, 32), (203, 0), (204, 16)])
def test_large_continuous_and_tied_tensors_in_the_forms_for_very_large_tensors(ctx_wide, seed, storage):
    """Two tensors of 0.6 to 1.5 M elements per batch -- Laplace steps, and a handful of distinct values
    (with 16-bit storage: residuals that are multiples of the format's unit, the case in which a
    sixteen-wave form of the per-bucket totals once gave a wrong centre) -- through the sixteen-wave,
    one-bucket-per-workgroup kernels and several candidate lists, blob for blob against the oracle."""
    run_batch(ctx_wide, seed, storage)


def run_batch(ctx, seed, big):
    nbits, iters, flags, alpha, beta, cases = draw_batch(seed, big)
    what = f"seed {seed}: nbits {nbits}, iters {iters}, flags {flags}, alpha {alpha}, beta {beta}, sizes {[c[0].size for c in cases]}"
    print(what, flush=True)
    stored_bits = 32 if flags & O.FLAG_NO_QUANT else nbits
    dev = []
    for (Wp, W, m, v) in cases:
        blob = torch.zeros(X.excp_blob_bound(W.size, stored_bits), dtype=torch.uint8, device="cuda")
        Wd = w_to_dev(Wp, flags)
        dev.append((Wd, w_to_dev(W, flags), torch.from_numpy(m).cuda(), torch.from_numpy(v).cuda(), blob,
                    torch.zeros_like(Wd)))
    ctx.excp_compress_tensors(dev, alpha, beta, nbits, iters, flags)
    rc, stats = ctx.excp_collect(check=False)
    assert rc == 0, what
    blobs, dec = [], []
    for c, t, st in zip(cases, dev, stats):
        ref = O.compress_step(*c, alpha, beta, nbits, iters, flags=flags)
        n = c[0].size
        assert (st.n_w, st.n_o) == (ref.n_w, ref.n_o), what
        blob = t[4][:int(st.blob_bytes)].cpu().numpy().tobytes()
        assert blob == ref.blob, what
        assert bits(w_to_host(t[5], flags)).tobytes() == bits(ref.W_recon).tobytes(), what
        blobs.append(blob)
        dec.append((t[0], t[4], int(st.blob_bytes), n, torch.zeros_like(t[5]),
                    torch.empty(n, dtype=torch.float32, device="cuda"),
                    torch.empty(n, dtype=torch.float32, device="cuda")))
    # Alg. 2 from the blobs
    ctx.excp_decompress_tensors(dec)
    rc, _ = ctx.excp_collect(check=False)
    assert rc == 0, what
    for c, blob, d in zip(cases, blobs, dec):
        W2, m2, v2 = O.decompress_step(c[0], blob)
        assert bits(w_to_host(d[4], flags)).tobytes() == bits(W2).tobytes(), what
        assert d[5].cpu().numpy().tobytes() == m2.tobytes() and d[6].cpu().numpy().tobytes() == v2.tobytes(), what
    if flags & O.FLAG_NO_QUANT:
        return                                      # no codes, hence no per-element code tensors
    # the stored layout of Sec. 4.2
    items, bufs = [], []
    for c, t, st in zip(cases, dev, stats):
        n = c[0].size
        db = X.excp_dense_bytes(n, nbits)
        b = [torch.zeros(max(X.excp_head_bytes(nbits), 16), dtype=torch.uint8, device="cuda")] + \
            [torch.zeros(db + 16, dtype=torch.uint8, device="cuda") for _ in range(3)]
        bufs.append(b)
        items.append((t[4], int(st.blob_bytes), n, *b))
    ctx.excp_export_dense(items)
    rc, _ = ctx.excp_collect(check=False)
    assert rc == 0, what
    for c, blob, b in zip(cases, blobs, bufs):
        db = X.excp_dense_bytes(c[0].size, nbits)
        ref = O.export_dense(blob)
        for got, want in zip(b[1:], ref[1:]):
            assert got[:db].cpu().numpy().tobytes() == want.tobytes(), what
