"""The whole LLaMA-7B-shaped checkpoint exactly as bench.py runs it: bench.Workload (four flat input
arrays resident in HBM, one view per tensor), one prepared batch of all 291 tensors, a context whose
groups hold half the model plus the largest tensor (two tensor groups), the benchmark's parameters.

Every tensor is checked through properties that hold at any size, computed on the device by library
routines that share nothing with the kernels (exact order statistics, exact fp32 products, population
counts, the reconstruction where nothing was kept); Alg. 2 through the library must return the
reconstruction compress kept; and tensors of both groups and of every kind (attention, MLP, norm) are
compared with the oracle on the whole blob."""
import importlib.util
import os

import numpy as np
import pytest
import torch

import paper_2406_11257_amd as X
from paper_2406_11257_amd import synth
from oracle.pool import OraclePool
from test_gpu_models import PARAMS, check_tensor

pytestmark = pytest.mark.gpu
f32 = np.float32
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def popcount_u8(t: torch.Tensor) -> int:
    """Set bits in a uint8 device tensor."""
    x = t.to(torch.int32)
    x = (x & 0x55) + ((x >> 1) & 0x55)
    x = (x & 0x33) + ((x >> 2) & 0x33)
    x = (x & 0x0f) + (x >> 4)
    return int(x.sum(dtype=torch.int64))


def test_whole_7b_shaped_checkpoint_in_the_benchmark_configuration():
    torch.cuda.empty_cache()                             # (what earlier tests left in torch's allocator counts as used)
    free, _ = torch.cuda.mem_get_info()
    cfg = synth.config(3)
    N, max_n = cfg.total, max(t.n for t in cfg.tensors)
    group = N // 2 + max_n                              # bench.py's default: two tensor groups
    if free < 20 * N + 1.8 * N + 26.0 * group + (2 << 30):
        pytest.skip("needs the memory of the benchmark's workload")
    B = load_bench()
    dev = torch.device("cuda", 0)
    wl = B.Workload(3, "f32", dev, synth.NBITS)
    ctx = X.Context(max_n, group, device=dev)
    batch = ctx.prepare_compress(wl.tensors, 0)
    # oracle beside the device checks: tensors of the first and of the second group, of every kind
    names = [t.name for t in cfg.tensors]
    first_group = [i for i in range(len(names)) if wl.offs[i] + cfg.tensors[i].n <= group]
    picks = [1, 8,                                       # layer 0 q_proj (16.8 M), input_layernorm (4096): first group
             len(names) - 9, len(names) - 5, len(names) - 2]   # last layer: an attention matrix, an MLP matrix (45 M), the final norm
    assert picks[0] in first_group and picks[2] not in first_group
    with OraclePool(len(picks)) as pool:
        for i in sorted(picks, key=lambda i: -cfg.tensors[i].n):
            pool.submit(f"t{i}", [wl.view(k, i).cpu().numpy() for k in range(4)], PARAMS)
        ctx.excp_compress_tensors(batch, synth.ALPHA, synth.BETA, synth.NBITS, synth.LLOYD_ITERS, 0)
        rc, stats = ctx.excp_collect(check=False)
        assert rc == 0 and len(stats) == len(cfg.tensors)

        books_off = 80
        kept_w = kept_o = 0
        for i, (spec, st) in enumerate(zip(cfg.tensors, stats)):
            tag = f"tensor {i} ({spec.name}, {spec.n})"
            n = spec.n
            Wp, W, m, v, blob, What = wl.tensors[i]
            assert st.status == 0 and st.n == n and st.n_o <= st.n_w <= n, tag
            assert st.blob_bytes == X.excp_blob_size(n, st.n_w, st.n_o, synth.NBITS), tag
            kept_w += st.n_w
            kept_o += st.n_o
            # thresholds: exact order statistic, exact fp32 products
            d = W - Wp
            kth = torch.kthvalue(d.abs(), (n - 1) // 2 + 1).values.item()
            assert f32(kth).tobytes() == f32(st.median_abs_dw).tobytes(), tag
            mean64 = m.abs().double().sum().item() / n
            assert abs(st.abs_sum_m / n - mean64) <= 1e-12 * mean64, tag
            assert f32(st.t_w).tobytes() == (f32(synth.ALPHA) * f32(st.median_abs_dw)).tobytes(), tag
            assert f32(st.r_o).tobytes() == (f32(synth.BETA) * f32(st.mean_abs_m)).tobytes(), tag
            # header and bitmaps
            head = blob[:80].cpu().numpy()
            assert head[:4].tobytes() == b"EXCP" and int(head[16:24].view(np.uint64)[0]) == n, tag
            assert (int(head[24:32].view(np.uint64)[0]), int(head[32:40].view(np.uint64)[0])) == (st.n_w, st.n_o), tag
            off_bw = books_off + 3 * (1 << synth.NBITS) * 4
            words_w = (n + 63) // 64
            bm = blob[off_bw:off_bw + 8 * words_w]
            assert popcount_u8(bm) == st.n_w, tag
            off_bo = off_bw + 8 * (words_w + (words_w & 1))
            words_o = (st.n_w + 63) // 64
            assert popcount_u8(blob[off_bo:off_bo + 8 * words_o]) == st.n_o, tag
            # the keep decision, element by element, where the device's own fp32 routines leave no doubt
            # (a relative margin of 1e-6 around the threshold; inside it the oracle decides, below)
            r = float(st.t_w) / v.sqrt()                # fp32 tensor arithmetic
            sure_keep, sure_drop = d.abs() > r * (1 + 1e-6), d.abs() < r * (1 - 1e-6)
            shifts = torch.arange(8, device=dev, dtype=torch.int32)
            bits = ((bm[:, None].to(torch.int32) >> shifts) & 1).reshape(-1)[:n].bool()
            assert not (sure_keep & ~bits).any() and not (sure_drop & bits).any(), tag
            # reconstruction: untouched where nothing was kept, moved elsewhere by one of the fifteen centres
            assert torch.equal(What[~bits], Wp[~bits]), tag
            book_w = blob[books_off:books_off + 64].cpu().numpy().view(np.float32)
            delta = (What[bits] - Wp[bits]).abs().max().item() if st.n_w else 0.0
            assert delta <= np.abs(book_w).max() + 1e-7, tag      # (the sum is rounded at the weight's magnitude)
            del d, r, sure_keep, sure_drop, bits
        assert abs(kept_w / N - 0.345) < 0.01 and abs(kept_o / N - 0.0757) < 0.005

        # Alg. 2 through the library over the whole checkpoint returns what compress kept
        out = torch.empty(N, dtype=torch.float32, device=dev)
        ctx.excp_decompress_tensors([(wl.tensors[i][0], wl.tensors[i][4], int(stats[i].blob_bytes), cfg.tensors[i].n,
                                      out[wl.offs[i]:wl.offs[i] + cfg.tensors[i].n], None, None) for i in range(len(names))])
        rc, _ = ctx.excp_collect(check=False)
        assert rc == 0 and torch.equal(out, wl.flat[4])
        del out

        for i in picks:
            check_tensor(f"tensor {i} ({names[i]})", pool.result(f"t{i}"), stats[i], wl.tensors[i][4], wl.tensors[i][5])
        print(f"config 3 in two groups: {len(names)} tensors, kept {kept_w / N:.4f} / {kept_o / N:.4f}; "
              f"{[names[i] for i in picks]} identical to the oracle's", flush=True)
    ctx.close()
