#!/usr/bin/env python3
"""Throughput of the ExCP compress step on one MI355X.

A "step" is one pass of the whole hot path over one synthetic checkpoint: residual, exact
thresholds, joint masks + compaction, k-means codebooks (10 Lloyd iterations), code packing and the
reconstructed weights kept for the next checkpoint -- for every tensor of the model, with W_prev,
W, m and v already resident in HBM.  The workload is the LLaMA-7B-shaped checkpoint (291 tensors,
6.74e9 parameters) when it fits on the device, otherwise the largest Pythia-shaped one that does.

Prints ONE JSON line (metric, value, roofline of the dominant kernel, CPU-oracle baseline).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def stage_bytes_per_param(p_w, p_o, nbits, iters, wb=4.0):
    """Algorithmic HBM bytes per parameter of each kernel stage (what the method must move); wb = bytes
    of one stored weight (4, or 2 for fp16 / bf16 checkpoints)."""
    s = p_w + 2.0 * p_o
    bitmaps = 0.125 * (1.0 + p_w)
    return {
        "stats_stream": 2.0 * wb + 4.0,                    # read W_prev, W, m
        "mask_slots": 2.0 * wb + 8.0 + 0.125 + 4.0 * s,    # read all four arrays; write keep bitmap + survivor slots
        "mask_gather": 8.0 * s + 0.25 * p_w,               # slots -> dense survivor arrays; local M_o bits -> bitmap_o
        "km_count": 4.0 * s,                               # read the survivors, count per bucket
        "km_scatter": 8.0 * s,                             # read the survivors, write them bucket by bucket
        "km_bucket_stats": 4.0 * s,                        # read the partitioned survivors once
        "assign_pack": 4.0 * s + s * nbits / 8.0,          # read survivors, write codes
        "decode_main": wb + bitmaps + s * nbits / 8.0 + wb,     # read W_prev, bitmaps, codes; write W_hat
    }


def step_bytes_per_param(p_w, p_o, wb=4.0):
    """Step-level accounting used for the '% of HBM roofline' headline: 32.2 + 58.5 s (+ 8 for W_hat) for
    fp32 weights; of the 32.2, sixteen bytes are the two passes over W_prev and W, and the 8 are W_prev
    read and W_hat written: those scale with the stored weight size."""
    s = p_w + 2.0 * p_o
    return 32.2 - 16.0 * (1.0 - wb / 4.0) + 58.5 * s + 8.0 * wb / 4.0


STAGE_KERNEL = {"stats_stream": "k_stats_stream<false>", "mask_slots": "k_mask_slots<false,false>", "mask_gather": "k_mask_gather",
                "km_count": "k_km_count", "km_scatter": "k_km_scatter", "km_bucket_stats": "k_km_bucket_stats<4u,4u>",
                "assign_pack": "k_assign_pack", "decode_main": "k_decode_main<false>"}


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` from the committed counter summary (profiles/hbm_traffic.txt:
    lines 'traffic <workload> <kernel> <fetch bytes> <write bytes>', already scaled by the copy-kernel
    calibration), or None when that kernel / workload has not been measured."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.txt")) as f:
            for line in f:
                p = line.split()
                if len(p) == 5 and p[0] == "traffic" and p[1] == workload and p[2] == kernel:
                    return float(p[3]) + float(p[4])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=-1, help="workload config id (default: largest that fits)")
    ap.add_argument("--groups", type=int, default=2, help="tensor groups a large checkpoint is processed in")
    ap.add_argument("--weights", choices=("f32", "f16", "bf16"), default="f32",
                    help="storage of W_prev, W and W_hat (the headline workload is f32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2406_11257_amd as X
    from paper_2406_11257_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda", 0)
    free, total_mem = torch.cuda.mem_get_info()
    alpha, beta, nbits, iters = synth.ALPHA, synth.BETA, synth.NBITS, synth.LLOYD_ITERS
    wdtype = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[args.weights]
    wflags = {"f32": 0, "f16": X.EXCP_FLAG_W_F16, "bf16": X.EXCP_FLAG_W_BF16}[args.weights]
    wb = 4.0 if args.weights == "f32" else 2.0

    def need_bytes(cfg, group):
        N = cfg.total
        return 20 * N + 1.8 * N + 26.0 * group + (2 << 30)   # inputs + W_hat, blobs, workspace, slack

    cid = args.config
    if cid < 0:
        for cand in (3, 2, 1, 0):
            cfg = synth.config(cand)
            if need_bytes(cfg, cfg.total // args.groups + max(t.n for t in cfg.tensors)) < free:
                cid = cand
                break
    cfg = synth.config(cid)
    N = cfg.total
    max_n = max(t.n for t in cfg.tensors)
    # tensors are processed in groups that share one workspace; fewer groups mean fewer launches, more
    # groups a smaller workspace.  N / ngroups + the largest tensor guarantees at most ngroups groups.
    group = min(N, N // args.groups + max_n) if N > (1 << 30) else N
    print(f"[bench] workload config {cid} ({cfg.name}): {len(cfg.tensors)} tensors, {N} params; "
          f"free HBM {free / 2**30:.1f} GiB", file=sys.stderr, flush=True)

    # ---- inputs resident in HBM: four flat arrays, one view per tensor -------------------------
    t0 = time.time()
    flat = [torch.empty(N, dtype=wdtype if k in (0, 1, 4) else torch.float32, device=dev)
            for k in range(5)]                                                    # Wp, W, m, v, W_hat
    offs, o = [], 0
    for i, spec in enumerate(cfg.tensors):
        Wp, W, m, v = synth.torch_draw_tensor(cid, i, spec, dev)
        for buf, src in zip(flat, (Wp, W, m, v)):
            buf[o:o + spec.n].copy_(src)
        del Wp, W, m, v
        offs.append(o)
        o += spec.n
    torch.cuda.synchronize()
    print(f"[bench] inputs drawn on the device in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)

    caps = [X.excp_blob_bound(t.n, nbits) for t in cfg.tensors]
    boffs = np.concatenate([[0], np.cumsum(caps)]).astype(np.int64)
    blob_flat = torch.empty(int(boffs[-1]), dtype=torch.uint8, device=dev)
    ctx = X.Context(max_n, group, device=dev)
    tensors = []
    for i, spec in enumerate(cfg.tensors):
        a, b = offs[i], offs[i] + spec.n
        tensors.append((flat[0][a:b], flat[1][a:b], flat[2][a:b], flat[3][a:b],
                        blob_flat[int(boffs[i]):int(boffs[i + 1])], flat[4][a:b]))

    # the argument array is built once: the tensors of a training job stay where they are between
    # checkpoints, and a C caller would hold such an array anyway
    batch = ctx.prepare_compress(tensors, wflags)

    def step():
        ctx.excp_compress_tensors(batch, alpha, beta, nbits, iters, wflags)
        return ctx.excp_collect()[1]

    for _ in range(args.warmup):
        stats = step()
    ctx.excp_set_profiling(True)
    stage_tot = {}
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_host = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        stats = step()
        for k, (ms, launches) in ctx.stage_times().items():
            a = stage_tot.setdefault(k, [0.0, 0])
            a[0] += ms
            a[1] += launches
    ev1.record()
    torch.cuda.synchronize()
    host_ms = (time.perf_counter() - t_host) * 1e3
    dev_ms = ev0.elapsed_time(ev1)
    ms_per_step = max(host_ms, dev_ms) / args.steps
    ctx.excp_set_profiling(False)

    # sanity of the last step (not timed): every tensor fine, sizes equal the closed form of the layout
    for spec, st_ in zip(cfg.tensors, stats):
        assert st_.status == 0 and st_.n == spec.n and st_.n_o <= st_.n_w <= st_.n
        assert st_.blob_bytes == X.excp_blob_size(spec.n, st_.n_w, st_.n_o, nbits)
    n_w = sum(s.n_w for s in stats)
    n_o = sum(s.n_o for s in stats)
    blob_bytes = sum(s.blob_bytes for s in stats)
    p_w, p_o = n_w / N, n_o / N
    params_per_s = N / (ms_per_step * 1e-3)

    # ---- roofline of the dominant kernel ----------------------------------------------------------
    per_param = stage_bytes_per_param(p_w, p_o, nbits, iters, wb)
    stage_report = {}
    for k, (ms, launches) in stage_tot.items():
        if launches == 0:
            continue
        e = {"ms_per_step": ms / args.steps, "launches_per_step": launches / args.steps}
        if k in per_param:
            e["algorithmic_GB_per_step"] = per_param[k] * N / 1e9
            e["achieved_GBs"] = per_param[k] * N / 1e9 / (ms / args.steps * 1e-3)
        stage_report[k] = e
    dominant = max((k for k in stage_report if k in per_param), key=lambda k: stage_report[k]["ms_per_step"])
    d = stage_report[dominant]
    roofline = {"bound": "hbm", "kernel": STAGE_KERNEL[dominant], "achieved": d["achieved_GBs"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": d["achieved_GBs"] / HBM_PEAK_GBS,
                "traffic": measured_traffic(STAGE_KERNEL[dominant], cfg.name),
                "avg_launch_ms": d["ms_per_step"] / d["launches_per_step"],
                "algorithmic_bytes_per_launch": per_param[dominant] * N / d["launches_per_step"],
                "algorithmic_bytes_per_param": per_param[dominant]}
    step_bytes = step_bytes_per_param(p_w, p_o, wb) * N
    step_frac = step_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9)

    # ---- decompress (Alg. 2) timing, reported beside the headline --------------------------------
    dec = [(flat[0][offs[i]:offs[i] + spec.n], tensors[i][4], int(stats[i].blob_bytes), spec.n,
            flat[4][offs[i]:offs[i] + spec.n], None, None)
           for i, spec in enumerate(cfg.tensors)]
    dec = ctx.prepare_decompress(dec)
    ctx.excp_decompress_tensors(dec); ctx.excp_collect()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(max(1, args.steps)):
        ctx.excp_decompress_tensors(dec)
        ctx.excp_collect()
    torch.cuda.synchronize()
    dec_ms = (time.perf_counter() - t1) * 1e3 / max(1, args.steps)

    # one plain copy of known size (1 GiB read + 1 GiB written): calibrates profiler byte counters
    probe = min(N * int(wb), 1 << 30) & ~15
    ctx.excp_copy_probe(flat[4], flat[0], probe)
    torch.cuda.synchronize()
    # the rate of a plain device-to-device copy on this GPU (torch's own copy kernel over up to 16 GiB):
    # what mixed read + write traffic reaches in practice, as a reference next to the 8 TB/s nominal peak
    cbytes = min(N * int(wb), 16 << 30)
    csrc, cdst = flat[0].view(torch.uint8)[:cbytes], flat[4].view(torch.uint8)[:cbytes]
    cdst.copy_(csrc)
    ce0, ce1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ce0.record()
    for _ in range(3):
        cdst.copy_(csrc)
    ce1.record()
    torch.cuda.synchronize()
    copy_GBs = 2.0 * cbytes * 3 / (ce0.elapsed_time(ce1) * 1e-3) / 1e9

    # ---- Alg. 3: a chain of 8 checkpoints in one pass (the same blob eight times: a valid chain) ------
    chain_len = 8
    chains = [(flat[0][offs[i]:offs[i] + spec.n], [tensors[i][4]] * chain_len, [int(stats[i].blob_bytes)] * chain_len,
               flat[4][offs[i]:offs[i] + spec.n], None, None) for i, spec in enumerate(cfg.tensors)]
    chains = ctx.prepare_chain(chains)
    ctx.excp_reconstruct_chain(chains); ctx.excp_collect()
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    for _ in range(max(1, args.steps)):
        ctx.excp_reconstruct_chain(chains)
        ctx.excp_collect()
    torch.cuda.synchronize()
    chain_ms = (time.perf_counter() - t4) * 1e3 / max(1, args.steps)

    # ---- CPU oracle on a bounded sample of the same workload -----------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle as O
        budget_elems = 16_000_000
        big = [i for i in range(len(cfg.tensors)) if cfg.tensors[i].n >= 1_000_000] or list(range(len(cfg.tensors)))
        pick = min(big, key=lambda i: (cfg.tensors[i].n, i))
        a, b = offs[pick], offs[pick] + min(cfg.tensors[pick].n, budget_elems)
        host = [(f[a:b].view(torch.int16).cpu().numpy().view(np.uint16) if f.dtype == torch.bfloat16
                 else f[a:b].cpu().numpy()) for f in flat[:4]]
        t2 = time.perf_counter()
        ref = O.compress_step(*host, alpha, beta, nbits, iters, flags=wflags)
        cpu_s = time.perf_counter() - t2
        cpu = {"value": (b - a) / cpu_s, "unit": "params/s", "cores": 1, "kind": "oracle",
               "sample": f"first {b - a} elements of tensor {pick} ({cfg.tensors[pick].name}) of the same "
                         f"checkpoint, {cpu_s:.1f} s; numpy, single thread; host has {os.cpu_count()} cores",
               "keep_fractions": [ref.n_w / (b - a), ref.n_o / (b - a)]}
        # the library on the same sample (untimed): its blob must be the oracle's, byte for byte
        sblob = torch.empty(X.excp_blob_bound(b - a, nbits), dtype=torch.uint8, device=dev)
        ctx.excp_compress_tensors([(flat[0][a:b], flat[1][a:b], flat[2][a:b], flat[3][a:b], sblob, None)],
                                  alpha, beta, nbits, iters, wflags)
        sst = ctx.excp_collect()[1][0]
        cpu["gpu_blob_identical"] = bool(sst.blob_bytes == len(ref.blob) and
                                         sblob[:int(sst.blob_bytes)].cpu().numpy().tobytes() == ref.blob)
        del sblob

    # ---- Alg. 2 with all three outputs (overwrites the m and v inputs: nothing needs them any more) ----
    dec3 = [(flat[0][offs[i]:offs[i] + spec.n], tensors[i][4], int(stats[i].blob_bytes), spec.n,
             flat[4][offs[i]:offs[i] + spec.n], flat[2][offs[i]:offs[i] + spec.n], flat[3][offs[i]:offs[i] + spec.n])
            for i, spec in enumerate(cfg.tensors)]
    dec3 = ctx.prepare_decompress(dec3)
    ctx.excp_decompress_tensors(dec3); ctx.excp_collect()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    for _ in range(max(1, args.steps)):
        ctx.excp_decompress_tensors(dec3)
        ctx.excp_collect()
    torch.cuda.synchronize()
    dec3_ms = (time.perf_counter() - t3) * 1e3 / max(1, args.steps)

    # ---- the stored layout of Sec. 4.2: export of the per-element code tensors, and Alg. 2 from them ----
    hb = X.excp_head_bytes(nbits)
    doffs, dtot = [], 0
    for spec in cfg.tensors:
        doffs.append(dtot)
        dtot += (X.excp_dense_bytes(spec.n, nbits) + 15) & ~15
    dense = [torch.empty(max(dtot, 16), dtype=torch.uint8, device=dev) for _ in range(3)]
    heads = torch.empty((len(cfg.tensors), (hb + 15) & ~15), dtype=torch.uint8, device=dev)
    dslice = lambda k, i: dense[k][doffs[i]:doffs[i] + X.excp_dense_bytes(cfg.tensors[i].n, nbits)]
    exp = [(tensors[i][4], int(stats[i].blob_bytes), spec.n, heads[i], dslice(0, i), dslice(1, i), dslice(2, i))
           for i, spec in enumerate(cfg.tensors)]
    imp = [(flat[0][offs[i]:offs[i] + spec.n], heads[i], hb, spec.n, dslice(0, i), dslice(1, i), dslice(2, i),
            flat[4][offs[i]:offs[i] + spec.n], flat[2][offs[i]:offs[i] + spec.n], flat[3][offs[i]:offs[i] + spec.n])
           for i, spec in enumerate(cfg.tensors)]
    dense_ms = {}
    for name, call, arg in (("export", ctx.excp_export_dense, ctx.prepare_export_dense(exp)),
                            ("decompress", ctx.excp_decompress_dense, ctx.prepare_decompress_dense(imp))):
        call(arg); ctx.excp_collect()
        torch.cuda.synchronize()
        t5 = time.perf_counter()
        for _ in range(max(1, args.steps)):
            call(arg)
            ctx.excp_collect()
        torch.cuda.synchronize()
        dense_ms[name] = (time.perf_counter() - t5) * 1e3 / max(1, args.steps)
    dense_bytes_total = len(cfg.tensors) * hb + 3 * sum(X.excp_dense_bytes(spec.n, nbits) for spec in cfg.tensors)

    out = {
        "metric": "checkpoint params compressed/sec and % of HBM roofline, 7B-shaped step",
        "value": params_per_s, "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {cid}: {cfg.name}-shaped checkpoint, {len(cfg.tensors)} tensors, {N} fp32 "
                               f"params x (W_prev, W, m, v) resident in HBM, weights stored as {args.weights}; alpha={alpha}, beta={beta}, nbits={nbits}, "
                               f"{iters} Lloyd iterations; W_hat emitted",
                   "params": N, "tensors": len(cfg.tensors), "group_elems": group},
        "state_GBs": (8.0 + 2.0 * wb) * N / (ms_per_step * 1e-3) / 1e9,
        "hbm_roofline_pct_step": 100.0 * step_frac,
        "step_algorithmic_bytes_per_param": step_bytes_per_param(p_w, p_o, wb),
        "keep_fractions": {"p_w": p_w, "p_o": p_o},
        "compression_ratio": (8.0 + wb) * N / blob_bytes,
        "decompress_ms": dec_ms, "decompress_params_per_s": N / (dec_ms * 1e-3),
        "decompress_with_moments_ms": dec3_ms,
        "reconstruct_chain_ms": {"checkpoints": chain_len, "ms": chain_ms, "one_by_one_ms": chain_len * dec_ms},
        "dense_layout": {"bytes": dense_bytes_total, "ratio": (8.0 + wb) * N / dense_bytes_total,
                         "export_ms": dense_ms["export"], "decompress_with_moments_ms": dense_ms["decompress"]},
        "workspace_GB": ctx.workspace_bytes / 1e9,
        "roofline": dict(roofline, plain_copy_GBs_same_gpu=copy_GBs),
        "cpu_baseline": cpu,
        "stages": stage_report,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
