#!/usr/bin/env python3
"""Throughput of the ExCP compress step on one MI355X.

A "step" is one pass of the whole hot path over one synthetic checkpoint: residual, exact
thresholds, joint masks + compaction, k-means codebooks (10 Lloyd iterations), code packing and the
reconstructed weights kept for the next checkpoint -- for every tensor of the model, with W_prev,
W, m and v already resident in HBM.  The workload is the LLaMA-7B-shaped checkpoint (291 tensors,
6.74e9 parameters) when it fits on the device, otherwise the largest Pythia-shaped one that does.

Prints ONE JSON line: the metric, the roofline of the dominant kernel, three step-level byte
accountings (the bytes this design's passes must move -- the headline percentage --, the survey-time
formula, and the traffic the profiler measured), the CPU oracle on a bounded sample of the same
workload, and the step times of the other benchmark configurations (`other_configs`).
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def stage_bytes_per_param(p_w, p_o, nbits, iters, wb=4.0):
    """Algorithmic HBM bytes per parameter of each kernel stage of THIS design (what its passes must
    move); wb = bytes of one stored weight (4, or 2 for fp16 / bf16 checkpoints)."""
    s = p_w + 2.0 * p_o
    bitmaps = 0.125 * (1.0 + p_w)
    return {
        "stats_stream": 2.0 * wb + 4.0,                    # read W_prev, W, m
        "mask_slots": 2.0 * wb + 8.0 + 0.125 + 4.0 * s,    # read all four arrays; write keep bitmap + survivor slots
        "mask_gather": 8.0 * s + 0.25 * p_w,               # slots -> dense survivor arrays (counting the value buckets on the way); local M_o bits -> bitmap_o
        "km_scatter": 8.0 * s,                             # read the survivors, write them bucket by bucket
        "km_bucket_stats": 4.0 * s,                        # read the partitioned survivors once
        "assign_pack": 4.0 * s + s * nbits / 8.0,          # read survivors, write codes
        "decode_main": wb + bitmaps + s * nbits / 8.0 + wb,     # read W_prev, bitmaps, codes; write W_hat
    }


def survey_bytes_per_param(p_w, p_o, wb=4.0):
    """The survey-time estimate 32.2 + 58.5 s (+ 8 for W_hat): it grants every Lloyd iteration a pass over
    the survivors (40 s), which the bucketed iterations of this design do not make.  Of the 32.2, sixteen
    bytes are the two passes over W_prev and W, and the 8 are W_prev read and W_hat written: those
    scale with the stored weight size."""
    s = p_w + 2.0 * p_o
    return 32.2 - 16.0 * (1.0 - wb / 4.0) + 58.5 * s + 8.0 * wb / 4.0


def stage_kernels(weights):
    w16 = weights != "f32"
    return {"stats_stream": "k_stats_stream<true>" if w16 else "k_stats_stream<false>",
            "mask_slots": "k_mask_slots<false,true>" if w16 else "k_mask_slots<false,false>",
            "mask_gather": "k_mask_gather", "km_scatter": "k_km_scatter",
            "km_bucket_stats": "k_km_bucket_stats<16u,4u>" if w16 else "k_km_bucket_stats<4u,4u>",
            "assign_pack": "k_assign_pack", "decode_main": "k_decode_main16<false>" if w16 else "k_decode_main<false>"}


def kernel_sources_hash():
    """Hash of the kernel sources: the stamp that ties profiles/hbm_traffic.txt to the code it measured."""
    from paper_2406_11257_amd.rocprof_summary import sources_hash
    return sources_hash()


def measured_traffic(workload):
    """{kernel: (bytes fetched, bytes written) per launch} from the committed counter summary
    (profiles/hbm_traffic.txt: a line 'sources <hash>' naming the kernel sources it was measured on, then
    lines 'traffic <workload> <kernel> <fetch bytes> <write bytes>', already scaled by the copy-kernel
    calibration), and whether that stamp is the hash of the sources in this tree."""
    table, stamp = {}, None
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.txt")) as f:
            for line in f:
                p = line.split()
                if len(p) == 2 and p[0] == "sources":
                    stamp = p[1]
                if len(p) == 5 and p[0] == "traffic" and p[1] == workload:
                    table[p[2]] = (float(p[3]), float(p[4]))
    except OSError:
        pass
    return table, (stamp is not None and stamp == kernel_sources_hash())


class Workload:
    """A checkpoint resident in HBM: four flat input arrays, W_hat, one blob area, one view per tensor."""

    def __init__(self, cid, weights, dev, nbits):
        import numpy as np
        import torch
        import paper_2406_11257_amd as X
        from paper_2406_11257_amd import synth
        self.cid, self.weights = cid, weights
        self.cfg = cfg = synth.config(cid)
        self.N = N = cfg.total
        wdtype = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[weights]
        self.wflags = {"f32": 0, "f16": X.EXCP_FLAG_W_F16, "bf16": X.EXCP_FLAG_W_BF16}[weights]
        self.wb = 4.0 if weights == "f32" else 2.0
        self.flat = [torch.empty(N, dtype=wdtype if k in (0, 1, 4) else torch.float32, device=dev) for k in range(5)]
        self.offs, o = [], 0
        for i, spec in enumerate(cfg.tensors):
            Wp, W, m, v = synth.torch_draw_tensor(cid, i, spec, dev)
            for buf, src in zip(self.flat, (Wp, W, m, v)):
                buf[o:o + spec.n].copy_(src)
            del Wp, W, m, v
            self.offs.append(o)
            o += spec.n
        caps = [X.excp_blob_bound(t.n, nbits) for t in cfg.tensors]
        self.boffs = np.concatenate([[0], np.cumsum(caps)]).astype(np.int64)
        self.blob_flat = torch.empty(int(self.boffs[-1]), dtype=torch.uint8, device=dev)
        self.tensors = []
        for i, spec in enumerate(cfg.tensors):
            a, b = self.offs[i], self.offs[i] + spec.n
            self.tensors.append((self.flat[0][a:b], self.flat[1][a:b], self.flat[2][a:b], self.flat[3][a:b],
                                 self.blob_flat[int(self.boffs[i]):int(self.boffs[i + 1])], self.flat[4][a:b]))

    def view(self, k, i):
        return self.flat[k][self.offs[i]:self.offs[i] + self.cfg.tensors[i].n]


def time_compress(ctx, wl, params, steps, warmup, profile):
    """W warm-up steps, then K timed ones; a step = excp_compress_tensors over the whole checkpoint +
    excp_collect.  Returns ms per step (the larger of host clock and device events over the K steps),
    the last step's per-tensor stats and the per-stage times summed over the K steps."""
    import torch
    alpha, beta, nbits, iters = params
    # the argument array is built once: the tensors of a training job stay where they are between
    # checkpoints, and a C caller would hold such an array anyway
    batch = ctx.prepare_compress(wl.tensors, wl.wflags)

    def step():
        ctx.excp_compress_tensors(batch, alpha, beta, nbits, iters, wl.wflags)
        return ctx.excp_collect()[1]

    for _ in range(warmup):
        stats = step()
    if profile:
        ctx.excp_set_profiling(True)
    stage_tot = {}
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_host = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        stats = step()
        if profile:
            for k, (ms, launches) in ctx.stage_times().items():
                a = stage_tot.setdefault(k, [0.0, 0])
                a[0] += ms
                a[1] += launches
    ev1.record()
    torch.cuda.synchronize()
    host_ms = (time.perf_counter() - t_host) * 1e3
    dev_ms = ev0.elapsed_time(ev1)
    if profile:
        ctx.excp_set_profiling(False)
    return max(host_ms, dev_ms) / steps, stats, stage_tot


def accounting(wl, stats, ms_per_step, params, stage_tot=None, steps=1, traffic=None):
    """Keep fractions, throughput and the step-level byte accountings of one timed workload."""
    import paper_2406_11257_amd as X
    alpha, beta, nbits, iters = params
    N = wl.N
    for spec, st_ in zip(wl.cfg.tensors, stats):       # sanity of the last step (not timed)
        assert st_.status == 0 and st_.n == spec.n and st_.n_o <= st_.n_w <= st_.n
        assert st_.blob_bytes == X.excp_blob_size(spec.n, st_.n_w, st_.n_o, nbits)
    p_w, p_o = sum(s.n_w for s in stats) / N, sum(s.n_o for s in stats) / N
    per_param = stage_bytes_per_param(p_w, p_o, nbits, iters, wl.wb)
    own = sum(per_param.values())
    t = ms_per_step * 1e-3
    out = {"ms_per_step": ms_per_step, "params_per_s": N / t,
           "state_GBs": (8.0 + 2.0 * wl.wb) * N / t / 1e9,
           "keep_fractions": {"p_w": p_w, "p_o": p_o},
           "compression_ratio": (8.0 + wl.wb) * N / sum(s.blob_bytes for s in stats),
           "step_own_minimum_bytes_per_param": own,
           "hbm_roofline_pct_step": 100.0 * own * N / t / (HBM_PEAK_GBS * 1e9),
           "survey_formula_bytes_per_param": survey_bytes_per_param(p_w, p_o, wl.wb),
           "hbm_pct_step_survey_formula": 100.0 * survey_bytes_per_param(p_w, p_o, wl.wb) * N / t / (HBM_PEAK_GBS * 1e9)}
    if traffic is not None and stage_tot:
        # measured bytes of the large kernels (per launch, from the counter profile) x their launches per step
        table, fresh = traffic
        kern = stage_kernels(wl.weights)
        tot = 0.0
        for stage, k in kern.items():
            if k not in table or stage not in stage_tot:
                tot = None
                break
            tot += sum(table[k]) * stage_tot[stage][1] / steps
        ok = fresh and tot is not None
        out["hbm_actual_pct_step"] = 100.0 * tot / t / (HBM_PEAK_GBS * 1e9) if ok else None
        out["step_measured_bytes_per_param"] = tot / N if ok else None
        if not ok:
            out["traffic_note"] = ("profiles/hbm_traffic.txt was measured on other kernel sources than this tree's"
                                   if not fresh else "profiles/hbm_traffic.txt does not cover this workload")
    return out, per_param


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
    ap.add_argument("--only-step", action="store_true",
                    help="the compress steps and the copy probe only (for profiler runs)")
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
    alpha, beta, nbits, iters = params = (synth.ALPHA, synth.BETA, synth.NBITS, synth.LLOYD_ITERS)

    def need_bytes(cfg, group):
        N = cfg.total
        return 20 * N + 1.8 * N + 26.0 * group + (2 << 30)   # inputs + W_hat, blobs, workspace, slack

    def group_elems(cfg):
        # tensors are processed in groups that share one workspace; fewer groups mean fewer launches, more
        # groups a smaller workspace.  N / ngroups + the largest tensor guarantees at most ngroups groups.
        N, max_n = cfg.total, max(t.n for t in cfg.tensors)
        return min(N, N // args.groups + max_n) if N > (1 << 30) else N

    cid = args.config
    if cid < 0:
        for cand in (3, 2, 1, 0):
            if need_bytes(synth.config(cand), group_elems(synth.config(cand))) < free:
                cid = cand
                break
    cfg = synth.config(cid)
    N, max_n, group = cfg.total, max(t.n for t in cfg.tensors), group_elems(cfg)
    print(f"[bench] workload config {cid} ({cfg.name}): {len(cfg.tensors)} tensors, {N} params; "
          f"free HBM {free / 2**30:.1f} GiB", file=sys.stderr, flush=True)

    # ---- inputs resident in HBM: four flat arrays, one view per tensor -------------------------
    t0 = time.time()
    wl = Workload(cid, args.weights, dev, nbits)
    torch.cuda.synchronize()
    print(f"[bench] inputs drawn on the device in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    flat, offs, tensors, wb, wflags = wl.flat, wl.offs, wl.tensors, wl.wb, wl.wflags
    ctx = X.Context(max_n, group, device=dev)

    ms_per_step, stats, stage_tot = time_compress(ctx, wl, params, args.steps, args.warmup, True)
    traffic = measured_traffic(cfg.name)
    acct, per_param = accounting(wl, stats, ms_per_step, params, stage_tot, args.steps, traffic)
    p_w, p_o = acct["keep_fractions"]["p_w"], acct["keep_fractions"]["p_o"]

    # ---- roofline of the dominant kernel ----------------------------------------------------------
    kern = stage_kernels(args.weights)
    stage_report = {}
    for k, (ms, launches) in stage_tot.items():
        if launches == 0:
            continue
        e = {"ms_per_step": ms / args.steps, "launches_per_step": launches / args.steps}
        if k in per_param:
            e["algorithmic_GB_per_step"] = per_param[k] * N / 1e9
            e["achieved_GBs"] = per_param[k] * N / 1e9 / (ms / args.steps * 1e-3)
            if traffic[1] and kern[k] in traffic[0]:
                e["measured_GB_per_step"] = sum(traffic[0][kern[k]]) * launches / args.steps / 1e9
        stage_report[k] = e
    dominant = max((k for k in stage_report if k in per_param), key=lambda k: stage_report[k]["ms_per_step"])
    d = stage_report[dominant]
    roofline = {"bound": "hbm", "kernel": kern[dominant], "achieved": d["achieved_GBs"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": d["achieved_GBs"] / HBM_PEAK_GBS,
                "traffic": sum(traffic[0][kern[dominant]]) if traffic[1] and kern[dominant] in traffic[0] else None,
                "avg_launch_ms": d["ms_per_step"] / d["launches_per_step"],
                "algorithmic_bytes_per_launch": per_param[dominant] * N / d["launches_per_step"],
                "algorithmic_bytes_per_param": per_param[dominant]}

    # one plain copy of known size (1 GiB read + 1 GiB written): calibrates profiler byte counters
    probe = min(N * int(wb), 1 << 30) & ~15
    ctx.excp_copy_probe(flat[4], flat[0], probe)
    torch.cuda.synchronize()

    out = {
        "metric": "checkpoint params compressed/sec and % of HBM roofline, 7B-shaped step",
        "value": acct["params_per_s"], "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {cid}: {cfg.name}-shaped checkpoint, {len(cfg.tensors)} tensors, {N} fp32 "
                               f"params x (W_prev, W, m, v) resident in HBM, weights stored as {args.weights}; alpha={alpha}, beta={beta}, nbits={nbits}, "
                               f"{iters} Lloyd iterations; W_hat emitted",
                   "params": N, "tensors": len(cfg.tensors), "group_elems": group},
    }
    out.update({k: v for k, v in acct.items() if k not in ("ms_per_step", "params_per_s")})
    out["workspace_GB"] = ctx.workspace_bytes / 1e9
    if args.only_step:
        out["roofline"] = roofline
        out["stages"] = stage_report
        print(json.dumps(out))
        return

    def timed(call, arg, reps):
        call(arg); ctx.excp_collect()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(reps):
            call(arg)
            ctx.excp_collect()
        torch.cuda.synchronize()
        return (time.perf_counter() - t1) * 1e3 / reps

    reps = max(1, args.steps)
    # ---- decompress (Alg. 2) timing, reported beside the headline --------------------------------
    dec = ctx.prepare_decompress([(wl.view(0, i), tensors[i][4], int(stats[i].blob_bytes), spec.n, wl.view(4, i), None, None)
                                  for i, spec in enumerate(cfg.tensors)])
    dec_ms = timed(ctx.excp_decompress_tensors, dec, reps)

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
    chains = ctx.prepare_chain([(wl.view(0, i), [tensors[i][4]] * chain_len, [int(stats[i].blob_bytes)] * chain_len,
                                 wl.view(4, i), None, None) for i, spec in enumerate(cfg.tensors)])
    chain_ms = timed(ctx.excp_reconstruct_chain, chains, reps)

    # ---- CPU oracle on a bounded sample of the same workload -----------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, stats, params)

    # ---- the other benchmark configurations, same run, same context (before anything overwrites m and v) ----
    others = []
    if cid == 3 and args.weights == "f32":
        del dec, chains
        others = other_configs(ctx, wl, params, traffic)
        # (the 16-bit runs wrote their blobs where the fp32 ones were: one untimed step puts those back)
        _, stats, _ = time_compress(ctx, wl, params, 1, 0, False)

    # ---- Alg. 2 with all three outputs (overwrites the m and v inputs: nothing needs them any more) ----
    dec3 = ctx.prepare_decompress([(wl.view(0, i), tensors[i][4], int(stats[i].blob_bytes), spec.n,
                                    wl.view(4, i), wl.view(2, i), wl.view(3, i)) for i, spec in enumerate(cfg.tensors)])
    dec3_ms = timed(ctx.excp_decompress_tensors, dec3, reps)

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
    imp = [(wl.view(0, i), heads[i], hb, spec.n, dslice(0, i), dslice(1, i), dslice(2, i),
            wl.view(4, i), wl.view(2, i), wl.view(3, i)) for i, spec in enumerate(cfg.tensors)]
    dense_ms = {"export": timed(ctx.excp_export_dense, ctx.prepare_export_dense(exp), reps),
                "decompress": timed(ctx.excp_decompress_dense, ctx.prepare_decompress_dense(imp), reps)}
    dense_bytes_total = len(cfg.tensors) * hb + 3 * sum(X.excp_dense_bytes(spec.n, nbits) for spec in cfg.tensors)
    del dense, heads, exp, imp, dec3

    out.update({
        "decompress_ms": dec_ms, "decompress_params_per_s": N / (dec_ms * 1e-3),
        "decompress_with_moments_ms": dec3_ms,
        "reconstruct_chain_ms": {"checkpoints": chain_len, "ms": chain_ms, "one_by_one_ms": chain_len * dec_ms},
        "dense_layout": {"bytes": dense_bytes_total, "ratio": (8.0 + wb) * N / dense_bytes_total,
                         "export_ms": dense_ms["export"], "decompress_with_moments_ms": dense_ms["decompress"]},
        "roofline": dict(roofline, plain_copy_GBs_same_gpu=copy_GBs),
        "cpu_baseline": cpu,
        "other_configs": others,
        "stages": stage_report,
    })
    print(json.dumps(out))


def cpu_baseline(wl, stats, params):
    """The oracle, as it stands, on one full transformer layer of the same checkpoint (or, for a small
    model, on the whole of it), its tensors fanned out over the host's cores by a pool of worker
    processes; the library's blobs of those tensors (from the last timed step) must be the oracle's."""
    import numpy as np
    import torch
    from oracle.pool import OraclePool, workers
    alpha, beta, nbits, iters = params
    cfg = wl.cfg
    layer = [i for i, t in enumerate(cfg.tensors) if t.name.startswith("layers.0.")]
    picks = layer if wl.N > 200_000_000 else list(range(len(cfg.tensors)))
    nw = workers()
    par = dict(alpha=alpha, beta=beta, nbits=nbits, iters=iters, flags=wl.wflags)
    host = {}
    for i in picks:
        host[i] = [(wl.view(k, i).view(torch.int16).cpu().numpy().view(np.uint16) if wl.flat[k].dtype == torch.bfloat16
                    else wl.view(k, i).cpu().numpy()) for k in range(4)]
    with OraclePool(nw) as pool:
        t2 = time.perf_counter()
        for i in picks:
            pool.submit(f"b{i}", host[i], par)
        res = {i: pool.result(f"b{i}") for i in picks}
        cpu_s = time.perf_counter() - t2
    elems = sum(cfg.tensors[i].n for i in picks)
    same = all(int(stats[i].blob_bytes) == res[i]["nbytes"] and
               hashlib.sha256(wl.tensors[i][4][:int(stats[i].blob_bytes)].cpu().numpy()).hexdigest() == res[i]["blob_sha"]
               for i in picks)
    core_s = sum(r["seconds"] for r in res.values())
    what = "transformer layer 0" if picks is layer else "the whole checkpoint"
    return {"value": elems / cpu_s, "unit": "params/s", "cores": min(nw, len(picks)), "kind": "oracle",
            "sample": f"{what} of the same checkpoint: {len(picks)} tensors, {elems} parameters, one oracle process per "
                      f"tensor over {min(nw, len(picks))} host cores (numpy, one thread each): {cpu_s:.1f} s wall, "
                      f"{core_s:.1f} core-seconds = {elems / core_s / 1e6:.2f} M params/s per core; host has {os.cpu_count()} cores"
                      + ("; the embedding and the output matrix (131 M elements each) are left out: about 80 s of one "
                         "core apiece" if picks is layer and wl.cid == 3 else ""),
            "per_core_params_per_s": elems / core_s,
            "keep_fractions": [sum(r["n_w"] for r in res.values()) / elems, sum(r["n_o"] for r in res.values()) / elems],
            "gpu_blob_identical": bool(same)}


def other_configs(ctx, main_wl, params, traffic):
    """Step times of the other benchmark configurations in the same process and context: the Pythia-shaped
    checkpoints (configs 0, 1, 2), one cell of the chained configuration (config 4: 8 checkpoints of the
    410M shape, each compressed against the previous reconstruction, nbits 4, alpha 5e-5), and the
    7B-shaped checkpoint with the weights stored as fp16 / bf16."""
    import torch
    from paper_2406_11257_amd import synth
    dev = main_wl.flat[0].device
    alpha, beta, nbits, iters = params
    res = []

    def entry(name, wl, ms, stats):
        a, _ = accounting(wl, stats, ms, params)
        return {"config": name, "params": wl.N, "tensors": len(wl.cfg.tensors), "weights": wl.weights,
                "ms_per_step": ms, "params_per_s": a["params_per_s"], "state_GBs": a["state_GBs"],
                "keep_fractions": a["keep_fractions"], "compression_ratio": a["compression_ratio"],
                "hbm_roofline_pct_step": a["hbm_roofline_pct_step"],
                "hbm_pct_step_survey_formula": a["hbm_pct_step_survey_formula"]}

    for cid in (0, 1, 2):
        wl = Workload(cid, "f32", dev, nbits)
        ms, stats, _ = time_compress(ctx, wl, params, 10, 3, False)
        res.append(entry(f"config {cid}: {wl.cfg.name}-shaped step", wl, ms, stats))
        if cid == 1:
            # config 4: the same shape, chained.  Step t: W += Laplace(0, 1e-4) update, fresh moments,
            # compressed against the previous reconstruction, which the call replaces in place.
            wl.flat[4].copy_(wl.flat[0])                       # W_hat_0 = W_0
            wl.flat[1].copy_(wl.flat[0])                       # the walk of the true weights starts there too
            chain = [(wl.view(4, i), t[1], t[2], t[3], t[4], wl.view(4, i)) for i, t in enumerate(wl.tensors)]
            batch = ctx.prepare_compress(chain, 0)
            tot, stats4 = 0.0, None
            for step in range(1, 9):
                for i, spec in enumerate(wl.cfg.tensors):
                    Wp_s, W_s, m, v = synth.torch_draw_tensor(4, i, spec, dev, step=step)
                    wl.view(1, i).add_(W_s - Wp_s)
                    wl.view(2, i).copy_(m)
                    wl.view(3, i).copy_(v)
                    del Wp_s, W_s, m, v
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                ctx.excp_compress_tensors(batch, alpha, beta, nbits, iters, 0)
                stats4 = ctx.excp_collect()[1]
                tot += (time.perf_counter() - t1) * 1e3
            e = entry("config 4: chain of 8 pythia-410m-shaped checkpoints, nbits 4, alpha 5e-05 (mean of the 8 steps; "
                      "keep fractions of the last)", wl, tot / 8.0, stats4)
            res.append(e)
        del wl
        torch.cuda.empty_cache()
    # the 7B shape with 16-bit weights: the same values, narrowed
    for weights, dt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        wl = main_wl
        w16 = object.__new__(Workload)
        w16.cid, w16.weights, w16.cfg, w16.N, w16.offs, w16.boffs, w16.blob_flat = wl.cid, weights, wl.cfg, wl.N, wl.offs, wl.boffs, wl.blob_flat
        import paper_2406_11257_amd as X
        w16.wflags = X.EXCP_FLAG_W_F16 if weights == "f16" else X.EXCP_FLAG_W_BF16
        w16.wb = 2.0
        w16.flat = [wl.flat[0].to(dt), wl.flat[1].to(dt), wl.flat[2], wl.flat[3], torch.empty(wl.N, dtype=dt, device=dev)]
        w16.tensors = []
        for i, spec in enumerate(wl.cfg.tensors):
            a, b = wl.offs[i], wl.offs[i] + spec.n
            w16.tensors.append((w16.flat[0][a:b], w16.flat[1][a:b], w16.flat[2][a:b], w16.flat[3][a:b],
                                wl.tensors[i][4], w16.flat[4][a:b]))
        ms, stats, _ = time_compress(ctx, w16, params, 5, 2, False)
        res.append(entry(f"config 3: {wl.cfg.name}-shaped step, weights stored as {weights}", w16, ms, stats))
        del w16
        torch.cuda.empty_cache()
    return res


if __name__ == "__main__":
    main()
