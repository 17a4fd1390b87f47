#!/usr/bin/env python3
"""Benchmark of the batched DLRM-style forward pass on one MI355X.

A step is one rec_model_forward over one synthetic batch (offsets scan, fused
SLS over all tables, bottom FC stack, pairwise-dot interaction, top FC stack +
sigmoid), inputs already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload rmc2] [--sweep] [--sched]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X fp32 matrix, published

# Bytes the pooling kernel reads from and writes to memory per launch, from rocprofv3 L2 request
# counters, live in a JSON block of this tracked summary together with the hash of the kernel source
# they were taken with; a changed kernel source makes them void (reported as null).
SLS_COUNTER_PROFILE = os.path.join("profiles", "sls_kernel_rmc2_counters.md")
SLS_SOURCE = os.path.join("paper_2001_02772_amd", "csrc", "sls.hip")


def counted_sls_traffic(workload):
    """(bytes per launch or None, where it came from)."""
    import hashlib
    import re
    try:
        text = open(os.path.join(ROOT, SLS_COUNTER_PROFILE)).read()
        block = json.loads(re.search(r"```json\s*(\{.*?\})\s*```", text, re.S).group(1))
        sha = hashlib.sha256(open(os.path.join(ROOT, SLS_SOURCE), "rb").read()).hexdigest()
    except (OSError, AttributeError, ValueError):
        return None, f"{SLS_COUNTER_PROFILE}: not readable"
    if block.get("sls_hip_sha256") != sha:
        return None, f"{SLS_COUNTER_PROFILE}: taken with another version of {SLS_SOURCE}, void"
    return block.get("traffic_bytes_per_launch", {}).get(workload), SLS_COUNTER_PROFILE


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="rmc2", choices=["tiny", "rmc1", "rmc2", "rmc2-uniform", "rmc3", "wnd"])
    ap.add_argument("--batches", type=int, default=16, help="distinct pre-generated batches rotated through")
    ap.add_argument("--streams", type=int, default=4,
                    help="streams the timed steps rotate over (1 = one batch at a time)")
    ap.add_argument("--repeats", type=int, default=5, help="the timed block of --steps steps is run this often; the median is reported")
    ap.add_argument("--only-sls", action="store_true",
                    help="set-up, then only launches of the pooling kernel (workload's indices, then uniform ones): for counter runs")
    ap.add_argument("--only-per-batch-size", action="store_true",
                    help="set-up, then only the whole-forward runs at sub-batch sizes 16/64/256/1024: for kernel traces")
    ap.add_argument("--only-mfma", action="store_true",
                    help="only the bf16 FC layers of the MLP-dominated model at batch 1024 / 4096 / 16384: for counter runs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-batch-size", action="store_true",
                    help="skip the short runs at sub-batch sizes 16/64/256 (keeps every launch of a profile at full batch)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain device copies of 256 MiB (reference dispatches for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--h2d", action="store_true",
                    help="also time the steps with every batch's inputs copied from pinned host memory")
    ap.add_argument("--sched", action="store_true",
                    help="also tune the request batch size by hill climbing on latency-bounded throughput")
    ap.add_argument("--no-sweep", action="store_true", help="skip the query-size sweep that the rmc2 run includes by default")
    ap.add_argument("--sweep", action="store_true",
                    help="also replay 2000 lognormal-sized queries split into sub-batches of 16/64/256/1024")
    return ap.parse_args()


def sls_algorithmic_bytes(cfg, n_indices, B):
    """Bytes the pooling must move if nothing is cached: per lookup one row (4D) and one
    index (4); per bag one length (4) and one pooled row written (4D)."""
    return n_indices * (4 * cfg.D + 4) + cfg.T * B * (4 + 4 * cfg.D)


def time_steps(fn, steps, warmup, torch, repeats=1):
    for i in range(warmup):
        fn(i)
    out = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        torch.cuda.synchronize()
        out.append((time.perf_counter() - t0) / steps)
    return out[0] if repeats == 1 else out


def time_many(model, rec, reqs, probs, streams, steps, warmup, torch, repeats=1):
    """K forward passes enqueued by one library call, request i on stream i % S; seconds per step,
    one figure per repeat of the K-step block (each bracketed by a device synchronisation)."""
    pick = lambda n: ([reqs[i % len(reqs)] for i in range(n)], [probs[i % len(probs)] for i in range(n)])
    timed = rec.ForwardMany(model, *pick(steps), streams)
    if warmup > 0:
        rec.ForwardMany(model, *pick(warmup), streams, workspaces=timed.ws).launch()
    out = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        timed.launch()
        torch.cuda.synchronize()
        out.append((time.perf_counter() - t0) / steps)
    return out


def median(v):
    v = sorted(v)
    return v[len(v) // 2]


def event_time(fn, steps, warmup, torch):
    """Average device time per launch between two events on the launch stream."""
    for i in range(warmup):
        fn(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / steps


def cpu_baseline(cfg, batch):
    """The oracle as it stands, timed on this host: whole forward of one full batch."""
    import oracle
    from paper_2001_02772_amd import synth
    tables, idx = synth.compact_tables(cfg, batch)
    pb, pt = synth.mlp_params(cfg.bottom, 0), synth.mlp_params(cfg.top, 1)

    def oracle_forward(cfg, tables, batch, indices):
        st, p = oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, batch.dense, indices, batch.lengths,
                                     bf16=cfg.bf16, concat=cfg.interaction == "concat")
        assert st == oracle.OK
        return p

    # one GPU's share of the host is 16 cores whatever the host shows; use those (all of them on a smaller host)
    cores = min(16, os.cpu_count() or 1)
    oracle.set_threads(cores)
    oracle_forward(cfg, tables, batch, indices=idx)               # warm-up
    runs, t_begin = [], time.perf_counter()
    while len(runs) < 3 or time.perf_counter() - t_begin < 8.0:
        t0 = time.perf_counter()
        p_all = oracle_forward(cfg, tables, batch, indices=idx)
        runs.append(time.perf_counter() - t0)
    oracle.set_threads(1)
    singles, t_begin = [], time.perf_counter()
    while len(singles) < 1 or time.perf_counter() - t_begin < 4.0:
        t0 = time.perf_counter()
        oracle_forward(cfg, tables, batch, indices=idx)
        singles.append(time.perf_counter() - t0)
    mean = sum(runs) / len(runs)
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
    except OSError:
        pass
    return {"value": batch.B / mean, "unit": "samples/s", "cores": cores, "host_cpus": os.cpu_count(), "kind": "oracle",
            "cpu_model": cpu_model,
            "sample": f"one full {cfg.name} batch of {batch.B} samples, whole forward, repeated {len(runs)} times "
                      f"(about 8 s) on {cores} threads; value = mean rate",
            "best_value": batch.B / min(runs),
            "single_thread_value": batch.B / (sum(singles) / len(singles))}, p_all


def sls_roofline(cfg, rec, model_tables, dbs, host_batches, steps, warmup, torch, np, workload_name, min_launches=100):
    """The fused gather-and-pool kernel alone between two events on its launch stream, over the given
    batches.  `achieved` / `frac` count only bytes that cross the memory side of the L2s (request
    counters of a tracked profile, else the compulsory bytes a batch cannot avoid), so the fraction is
    an HBM fraction; the algorithmic rate, which counts every looked-up row whether or not a cache
    served it, is reported beside it."""
    V = cfg.T + 1
    offs = [rec.sls_offsets(d.lengths) for d in dbs]
    vecs = torch.empty((cfg.B, V, cfg.D), dtype=torch.float32, device="cuda")

    def sls_only(i):
        d = dbs[i % len(dbs)]
        rec.sls_forward_offsets(model_tables, d.indices, offs[i % len(dbs)], d.B, out=vecs[:, 1:, :],
                                out_stride_b=V * cfg.D, out_stride_t=cfg.D)

    steps = max(steps, min_launches)            # kernel-only timing is cheap: the full run never takes fewer than 100 launches
    sec = event_time(sls_only, steps, warmup, torch)
    used = [dbs[i % len(dbs)].n_indices for i in range(steps)]
    alg = float(np.mean([sls_algorithmic_bytes(cfg, n, cfg.B) for n in used]))
    # compulsory traffic: distinct rows one batch touches (x row bytes) + its indices, offsets and pooled rows
    hb = host_batches[0]
    off = np.concatenate([[0], np.cumsum(hb.lengths, dtype=np.int64)])
    distinct = int(sum(np.unique(hb.indices[off[t * cfg.B]:off[(t + 1) * cfg.B]]).size for t in range(cfg.T)))
    compulsory = distinct * 4 * cfg.D + hb.indices.size * 4 + cfg.T * cfg.B * (8 + 4 * cfg.D)
    traffic, source = counted_sls_traffic(workload_name)
    hbm_bytes = traffic if traffic else compulsory
    r = {"bound": "hbm", "kernel": "sls_kernel", "achieved": hbm_bytes / sec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": hbm_bytes / sec / 1e9 / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": source,
         "achieved_basis": ("bytes through the memory side of the L2s per launch (request counters)" if traffic else
                            "compulsory bytes per launch (distinct rows + indices + offsets + output): a lower bound, no valid counter figure"),
         "us_per_launch": sec * 1e6, "algorithmic_bytes_per_launch": alg,
         "achieved_algorithmic": alg / sec / 1e9, "frac_algorithmic": alg / sec / 1e9 / HBM_PEAK_GBS,
         "algorithmic_note": "every looked-up row counted once per lookup; includes rows served by L2, so it may exceed the HBM peak",
         "distinct_rows_per_batch": distinct, "compulsory_bytes_per_launch": compulsory}
    if traffic:
        r["cache_served_fraction"] = 1.0 - traffic / alg
    return r


def mfma_roofline(rec, synth, torch, steps, warmup, batches=(1024, 4096, 16384), workload="rmc3", min_launches=100):
    """The FC layers of an MLP-dominated model (rmc3 shape: 2560-1024-256-32 and 87-512-256-1; wnd shape:
    2048-1024-512-256-1; bf16 operands, fp32 accumulate) through rec_mlp_forward with resident random
    inputs: the first (widest) layer alone at several batch sizes and the stacks at the model's batch.
    Every figure is all-in: fp32 activations in, the bf16 copy, the matrix kernel(s), fp32 out."""
    cfg = synth.CONFIGS[workload]
    pb, pt = synth.mlp_params(cfg.bottom, 0), synth.mlp_params(cfg.top, 1)
    dev = lambda a: torch.from_numpy(a).cuda()
    Wb, bb = [rec.f32_to_bf16(dev(w)) for w in pb.W], [dev(v) for v in pb.b]
    Wt, bt = [rec.f32_to_bf16(dev(w)) for w in pt.W], [dev(v) for v in pt.b]
    first_W, first_b = (Wb, bb) if Wb else (Wt, bt)           # a model without a dense stack: its first predictor layer
    F, n1 = first_W[0].shape[1], first_W[0].shape[0]

    def run(Ws, bs, B, final_act, n):
        widths = [Ws[0].shape[1]] + [w.shape[0] for w in Ws]
        x = torch.randn((B, widths[0]), dtype=torch.float32, device="cuda")
        y = torch.empty((B, widths[-1]), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(256, rec.mlp_workspace_bytes(widths, B, rec.BF16)), dtype=torch.uint8, device="cuda")
        sec = event_time(lambda i: rec.mlp_forward(Ws, bs, x, rec.ACT_RELU, final_act, wdtype=rec.BF16, y=y, ldy=widths[-1],
                                                   workspace=ws), n, warmup, torch)
        fl = 2.0 * B * sum(widths[l] * widths[l + 1] for l in range(len(Ws)))
        return {"us": sec * 1e6, "flops": fl, "tflops": fl / sec / 1e12, "frac": fl / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS}

    steps = max(steps, min_launches)            # layer-only timing: the full run never takes fewer than 100 launches (a quarter at the largest batch)
    sweep = {str(B): run(first_W[:1], first_b[:1], B, rec.ACT_RELU, steps if B <= 4096 else max(20, steps // 4)) for B in batches}
    l1 = sweep[str(cfg.B)]
    zero = {"us": 0.0, "flops": 0.0, "tflops": 0.0, "frac": 0.0}
    bottom = run(Wb, bb, cfg.B, rec.ACT_RELU, steps) if Wb else zero
    top = run(Wt, bt, cfg.B, rec.ACT_SIGMOID, steps)
    both = {"us": bottom["us"] + top["us"], "flops": bottom["flops"] + top["flops"]}
    both["tflops"] = both["flops"] / both["us"] / 1e6
    both["frac"] = both["tflops"] / MFMA_BF16_PEAK_TFLOPS
    return {"bound": "mfma", "kernel": "prepare_bf16_kernel + gemm_ks_kernel (64x64 tiles) or gemm_bf16_kernel (128x128, 256x256 tiles)", "achieved": l1["tflops"],
            "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": l1["frac"], "traffic": None, "us_per_launch": l1["us"],
            "flops_per_launch": l1["flops"],
            "layer": f"{cfg.B}x{F} . ({n1}x{F})^T bf16 operands, fp32 accumulate; fp32 in and out through rec_mlp_forward",
            "batch_sweep": sweep, "stacks": {"bottom": bottom, "top": top, "both": both}}


def per_batch_size(cfg, model, host_batches, probs, ws, streams, a, torch, rec, synth, workload):
    """samples/s of the whole forward per sub-batch size (the batch sizes of the query-size sweep)."""
    per_b = {}
    for Bs in synth.SWEEP_BATCH_SIZES:
        if Bs > cfg.B or a.no_per_batch_size:
            continue
        subs = [workload.DeviceBatch(workload.slice_batch(host_batches[k % len(host_batches)], cfg.T, 0, Bs))
                for k in range(4)]

        def sub_step(i, subs=subs, Bs=Bs):
            d = subs[i % len(subs)]
            model.forward(d.dense, d.indices, d.lengths, Bs, prob=probs[0], workspace=ws)

        s1 = time_steps(sub_step, max(50, a.steps // 2), 10, torch)
        s = median(time_many(model, rec, subs, [probs[0][:Bs].clone() for _ in subs], streams, max(50, a.steps // 2), 10,
                             torch, repeats=3)) if a.streams > 1 else s1
        per_b[str(Bs)] = {"samples_per_s": Bs / s, "us_per_batch": s * 1e6,
                          "single_stream": {"samples_per_s": Bs / s1, "us_per_batch": s1 * 1e6}}
    return per_b


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the model is replicated and queries are split across GPUs with no communication).",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2001_02772_amd import rec, synth, workload
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    rec.lib()
    # the pool is created before anything else touches the device: streams created first are the
    # ones the runtime spreads over distinct hardware queues
    pool = rec.StreamPool(a.streams)
    streams = pool.streams
    if a.only_mfma:
        print(json.dumps({"mfma_roofline": mfma_roofline(rec, synth, torch, a.steps, a.warmup, min_launches=0)}))
        return
    cfg = synth.CONFIGS[a.workload]
    t_setup = time.perf_counter()
    model = workload.device_model(cfg)
    gen = synth.BatchGenerator(cfg)
    host_batches = [gen.batch(k) for k in range(a.batches)]
    dbs = [workload.DeviceBatch(b) for b in host_batches]
    probs = [torch.empty(cfg.B, dtype=torch.float32, device="cuda") for _ in dbs]
    ws = model.workspace(cfg.B)
    setup_s = time.perf_counter() - t_setup
    torch.cuda.synchronize()            # set-up (on torch's stream) is complete before the pool's streams start

    # the uniform-index control of the embedding-dominated model: same tables, same bag lengths' law
    uniform = None
    if cfg.name == "rmc2":
        ucfg = synth.CONFIGS["rmc2-uniform"]
        ugen = synth.BatchGenerator(ucfg)
        uhost = [ugen.batch(k) for k in range(4)]
        uniform = (ucfg, [workload.DeviceBatch(b) for b in uhost], uhost)

    if a.only_sls:
        out = {"roofline": sls_roofline(cfg, rec, model.tables, dbs, host_batches, a.steps, a.warmup, torch, np, cfg.name, min_launches=0)}
        if uniform:
            out["roofline_uniform"] = sls_roofline(uniform[0], rec, model.tables, uniform[1], uniform[2], a.steps, a.warmup,
                                                   torch, np, "rmc2-uniform", min_launches=0)
        if a.copy_calibration:
            out["copy_calibration"] = copy_calibration(cfg, model, rec, torch)
        print(json.dumps(out))
        return

    if a.only_per_batch_size:
        print(json.dumps({"per_batch_size": per_batch_size(cfg, model, host_batches, probs, ws, streams, a, torch, rec, synth,
                                                           workload)}))
        return

    def step(i):
        d = dbs[i % len(dbs)]
        model.forward(d.dense, d.indices, d.lengths, d.B, prob=probs[i % len(dbs)], workspace=ws)

    # Headline: K steps over S streams (request i on stream i % S), so that the latency-bound
    # kernels of one batch run in the gaps of another; the single-stream figure (one batch at a
    # time, the latency view) is reported next to it.  The K-step block is timed `repeats` times,
    # each between device synchronisations; the median is the reported figure.
    single_runs = time_steps(step, a.steps, a.warmup, torch, repeats=max(1, a.repeats))
    single_runs = single_runs if isinstance(single_runs, list) else [single_runs]
    sec_single = median(single_runs)
    lat = []                                   # one step at a time, enqueue to completion on the host clock
    for i in range(a.steps):
        t0 = time.perf_counter()
        step(i)
        torch.cuda.synchronize()
        lat.append(time.perf_counter() - t0)
    lat.sort()
    many_runs = (time_many(model, rec, dbs, probs, streams, a.steps, a.warmup, torch, repeats=max(1, a.repeats))
                 if a.streams > 1 else single_runs)
    sec = median(many_runs)
    value = cfg.B / sec

    roofline = sls_roofline(cfg, rec, model.tables, dbs, host_batches, a.steps, a.warmup, torch, np, cfg.name)
    sls_gbs = roofline["achieved_algorithmic"]

    # the two FC stacks timed alone (all their launches between two events): achieved FLOP/s.
    # (Through rec_mlp_forward with the caller's weights: inside the model the first predictor layer
    # of a dot-interaction model runs on a copy padded for aligned loads and is faster than here.)
    def stack_rate(Ws, bs, x, final_act):
        if not Ws:
            return None
        widths = [Ws[0].shape[1]] + [w.shape[0] for w in Ws]
        wd = rec.BF16 if cfg.bf16 else rec.F32
        y = torch.empty((cfg.B, widths[-1]), dtype=torch.float32, device="cuda")
        wsb = torch.empty(max(256, rec.mlp_workspace_bytes(widths, cfg.B, wd)), dtype=torch.uint8, device="cuda")
        sec_ = event_time(lambda i: rec.mlp_forward(Ws, bs, x, rec.ACT_RELU, final_act, wdtype=wd, y=y, ldy=widths[-1],
                                                    workspace=wsb), a.steps, a.warmup, torch)
        fl = 2.0 * cfg.B * sum(widths[l] * widths[l + 1] for l in range(len(Ws)))
        return {"widths": widths, "us": sec_ * 1e6, "flops": fl, "tflops": fl / sec_ / 1e12}

    peak_tf = MFMA_BF16_PEAK_TFLOPS if cfg.bf16 else MFMA_F32_PEAK_TFLOPS
    stacks = {"bottom": stack_rate(model.bottom_W, model.bottom_b, dbs[0].dense, rec.ACT_RELU),
              "top": stack_rate(model.top_W, model.top_b,
                                torch.randn((cfg.B, model.top_W[0].shape[1]), dtype=torch.float32, device="cuda"),
                                rec.ACT_SIGMOID)}
    both = [s for s in stacks.values() if s]
    stacks["total"] = {"us": sum(s["us"] for s in both), "flops": sum(s["flops"] for s in both),
                       "tflops": sum(s["flops"] for s in both) / sum(s["us"] for s in both) / 1e6,
                       "peak_tflops": peak_tf,
                       "frac": sum(s["flops"] for s in both) / sum(s["us"] for s in both) / 1e6 / peak_tf}

    per_b = per_batch_size(cfg, model, host_batches, probs, ws, streams, a, torch, rec, synth, workload)

    metric = ("samples/sec per batch size + SLS achieved HBM GB/s (RMC2-shaped, 1 GPU)" if cfg.name == "rmc2"
              else f"samples/sec per batch size ({cfg.name}-shaped, 1 GPU)")
    out = {"metric": metric,
           "value": value, "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
           "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if cfg.bf16 else "f32", "data": "synthetic",
           "config": {"workload": f"{cfg.name}-shaped DLRM forward", "batch": cfg.B, "tables": cfg.T, "rows": cfg.R,
                      "dim": cfg.D, "lookups_per_bag": f"U{{{cfg.len_lo}..{cfg.len_hi}}}", "indices": cfg.index_dist,
                      "bottom": list(cfg.bottom), "top": list(cfg.top), "interaction": cfg.interaction,
                      "distinct_batches": len(dbs), "streams": a.streams},
           "timing": {"repeats": len(many_runs), "ms_per_step_each_repeat": [r * 1e3 for r in many_runs],
                      "reported": "median over the repeats of the timed block of `steps` steps"},
           "single_stream": {"value": cfg.B / sec_single, "ms_per_step": sec_single * 1e3,
                             "ms_per_step_each_repeat": [r * 1e3 for r in single_runs],
                             "latency_ms_median": lat[len(lat) // 2] * 1e3, "latency_ms_min": lat[0] * 1e3},
           "sls_gbs": sls_gbs, "per_batch_size": per_b, "fc_stacks": stacks, "setup_s": setup_s}
    if cfg.bf16:
        # MLP-dominated workload: the dominant kernel is the first (widest) Dense-FC layer
        out["roofline"] = mfma_roofline(rec, synth, torch, a.steps, a.warmup, workload=cfg.name)
        out["sls_roofline"] = roofline
    else:
        out["roofline"] = roofline
    if uniform:
        out["roofline_uniform"] = sls_roofline(uniform[0], rec, model.tables, uniform[1], uniform[2], a.steps, a.warmup, torch,
                                               np, "rmc2-uniform")
        # the other target of this build: bf16 MFMA rate of the MLP-dominated model's FC layers
        out["mfma_roofline"] = mfma_roofline(rec, synth, torch, a.steps, a.warmup)

    if a.copy_calibration:
        out["copy_calibration"] = copy_calibration(cfg, model, rec, torch)

    if a.sweep or (cfg.name == "rmc2" and not a.no_sweep):
        # the query-size sweep workload (2000 lognormal-sized queries cut into sub-batches of 16/64/256/1024);
        # host-to-device columns only on request, they need pinned copies of the inputs
        out["query_sweep"] = query_sweep(cfg, model, gen, ws, torch, rec, synth, workload, np,
                                        h2d_queries=300 if (a.sweep or a.h2d) else 0)

    if a.h2d:
        out["h2d_inclusive"] = h2d_inclusive(cfg, model, host_batches, streams, a.steps, a.warmup, torch)

    if a.sched:
        out["batch_size_tuning"] = batch_size_tuning(cfg, model, gen, torch, rec, synth, workload, np,
                                                     pool_streams=streams if a.streams > 1 else None)
        if not a.no_cpu_baseline:
            out["offload_threshold_tuning"] = offload_threshold_tuning(
                cfg, out["batch_size_tuning"]["service_table_s"], gen, torch, rec, synth, workload, np)

    if not a.no_cpu_baseline:
        base, p_cpu = cpu_baseline(cfg, host_batches[0])
        out["cpu_baseline"] = base
        # the timed GPU path and the CPU baseline computed the same thing
        step(0)
        torch.cuda.synchronize()
        p_gpu = probs[0].cpu().numpy()
        out["max_abs_diff_vs_oracle"] = float(np.max(np.abs(p_gpu - p_cpu)))
    print(json.dumps(out))


def copy_calibration(cfg, model, rec, torch):
    """Reference dispatches of known size for checking memory counters:
    (1) the pooling kernel itself streaming a table once -- one table, bag i = rows 4i..4i+3
        (four lookups per bag keep it on sls_kernel, not on the short-bag kernel), so it reads n
        rows (+ n indices, n/4+1 offsets) and writes n/4 rows with the request pattern of the real run;
    (2) the runtime's device-to-device copy of 256 MiB."""
    n = min(cfg.R, 500_000) // 4 * 4
    nb = n // 4
    one = rec.Tables([model.tables.tensors[0]])
    idx = torch.arange(n, dtype=torch.int32, device="cuda")
    off = torch.arange(nb + 1, dtype=torch.int64, device="cuda") * 4
    dst_rows = torch.empty((nb, 1, cfg.D), dtype=torch.float32, device="cuda")
    for _ in range(3):
        rec.sls_forward_offsets(one, idx, off, nb, out=dst_rows, out_stride_b=cfg.D, out_stride_t=cfg.D)
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    return {"sls_as_copy": {"grid_threads": ((nb + 3) // 4) * 256, "read_bytes": n * (4 * cfg.D + 4) + 8 * (nb + 1),
                            "write_bytes": nb * 4 * cfg.D},
            "memcpy_d2d_bytes": int(src.numel())}


def query_sweep(cfg, model, gen, ws, torch, rec, synth, workload, np, h2d_queries=300):
    """2000 queries, sizes lognormal(4.5, 1.0) clipped to [1, 1000], each split into sub-batches
    of B and served one after another; latency = first enqueue to completion of the last.
    Inputs are resident on the device; for the first `h2d_queries` queries the replay is repeated with
    every sub-batch's inputs copied from pinned host memory first (the `with_h2d` figures)."""
    sizes = synth.lognormal_query_sizes(synth.MASTER_SEED, synth.SWEEP_QUERIES)
    pool = [gen.batch(100 + k, B=1000) for k in range(8)]           # item pools to cut queries from
    res = {}
    prob = torch.empty(1024, dtype=torch.float32, device="cuda")
    rank = lambda srt, p: float(srt[max(0, int(np.ceil(p * len(srt))) - 1)])
    stats = lambda lat, total, n_items: {"samples_per_s": float(n_items / total), "latency_ms_p50": rank(np.sort(lat), 0.50) * 1e3,
                                         "latency_ms_p95": rank(np.sort(lat), 0.95) * 1e3,
                                         "latency_ms_p99": rank(np.sort(lat), 0.99) * 1e3}
    for Bs in synth.SWEEP_BATCH_SIZES:
        # pre-stage every sub-batch on the device (inputs resident, as for the headline number)
        host, staged = [], []
        for q, n in enumerate(sizes.tolist()):
            src = pool[q % len(pool)]
            parts = [workload.slice_batch(src, cfg.T, s, c) for s, c in rec.split_query(n, Bs)]
            staged.append([workload.DeviceBatch(b) for b in parts])
            if q < h2d_queries:
                host.append([(torch.from_numpy(b.dense).pin_memory(), torch.from_numpy(b.indices).pin_memory(),
                              torch.from_numpy(b.lengths).pin_memory()) for b in parts])
        lat = np.empty(len(staged))
        for warm in (True, False):
            torch.cuda.synchronize()
            t_all = time.perf_counter()
            for q, subs in enumerate(staged):
                t0 = time.perf_counter()
                for d in subs:
                    model.forward(d.dense, d.indices, d.lengths, d.B, prob=prob, workspace=ws)
                torch.cuda.synchronize()
                lat[q] = time.perf_counter() - t0
                if warm and q >= 50:
                    break
            total = time.perf_counter() - t_all
        res[str(Bs)] = stats(lat, total, sizes.sum())
        # the same replay with the inputs of every sub-batch coming from (pinned) host memory
        nq = len(host)
        lat_d, lat_h = np.empty(nq), np.empty(nq)
        for mode, out_lat in ((("dev", lat_d), ("h2d", lat_h)) if nq else ()):
            torch.cuda.synchronize()
            t_all = time.perf_counter()
            for q in range(nq):
                t0 = time.perf_counter()
                for d, (hd, hi, hl) in zip(staged[q], host[q]):
                    if mode == "h2d":
                        d.dense.copy_(hd, non_blocking=True)
                        d.indices.copy_(hi, non_blocking=True)
                        d.lengths.copy_(hl, non_blocking=True)
                    model.forward(d.dense, d.indices, d.lengths, d.B, prob=prob, workspace=ws)
                torch.cuda.synchronize()
                out_lat[q] = time.perf_counter() - t0
            tot = time.perf_counter() - t_all
            res[str(Bs)]["first_%d_queries_%s" % (nq, "resident" if mode == "dev" else "with_h2d")] = stats(out_lat, tot, sizes[:nq].sum())
        del staged, host
    return res


# p95 latency targets per model, ms (Table II, "medium"); low / high = 0.5x / 1.5x (Section V)
TABLE_II_TARGET_MS = {"rmc1": 100.0, "rmc2": 400.0, "rmc2-uniform": 400.0, "rmc3": 100.0}


def h2d_inclusive(cfg, model, host_batches, streams, steps, warmup, torch):
    """The same steps with every batch's inputs (dense, indices, lengths) copied from pinned host
    memory on the stream that then runs the forward: the rate a caller with host-resident inputs
    sees.  Never the headline value."""
    ext = [torch.cuda.ExternalStream(s.cuda_stream) for s in streams]
    pinned = [(torch.from_numpy(b.dense).pin_memory(), torch.from_numpy(b.indices).pin_memory(),
               torch.from_numpy(b.lengths).pin_memory()) for b in host_batches]
    n_max = max(b.indices.size for b in host_batches)
    slots = [(torch.empty((cfg.B, cfg.F), dtype=torch.float32, device="cuda"),
              torch.empty(n_max, dtype=torch.int32, device="cuda"),
              torch.empty(cfg.T * cfg.B, dtype=torch.int32, device="cuda"),
              torch.empty(cfg.B, dtype=torch.float32, device="cuda"),
              torch.empty(model.workspace_bytes(cfg.B), dtype=torch.uint8, device="cuda")) for _ in ext]
    nbytes = sum(d.numel() * 4 + i.numel() * 4 + l.numel() * 4 for d, i, l in pinned) / len(pinned)

    def run(n):
        for i in range(n):
            k = i % len(ext)
            d, ix, ln = pinned[i % len(pinned)]
            dd, di, dl, prob, ws = slots[k]
            with torch.cuda.stream(ext[k]):
                dd.copy_(d, non_blocking=True)
                di[: ix.numel()].copy_(ix, non_blocking=True)
                dl.copy_(ln, non_blocking=True)
                model.forward(dd, di[: ix.numel()], dl, cfg.B, prob=prob, workspace=ws)

    run(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    return {"value": cfg.B / sec, "unit": "samples/s", "ms_per_step": sec * 1e3, "host_bytes_per_step": nbytes,
            "host_to_device_gbs": nbytes / sec / 1e9}


def batch_size_tuning(cfg, model, gen, torch, rec, synth, workload, np,
                      sla_ms=(0.25, 0.5, 1.0, 5.0), live_load=0.8, pool_streams=None):
    """Batch-size hill climb on latency-bounded throughput (Sections III-B, IV-C), then an open-loop
    check of the prediction with Poisson arrivals on the device (Section III-C).

    1. Request service time t[b]: one burst replay in which every query is a single request of b
       items; consecutive completion timestamps give t[b] (median over repeats).  Measured for
       b = 1..32, every 8 up to 256 and every 32 up to 1024; linear in between.
    2. For each latency target: max query rate with p95 <= target for batch sizes 1, 2, 4 .. 1024,
       and the batch size the hill climb keeps.
    3. Live: the trace replayed at `live_load` x the predicted rate with the chosen batch size."""
    grid = sorted(set(list(range(1, 33)) + list(range(40, 257, 8)) + list(range(288, 1025, 32))))
    grid = [b for b in grid if b <= 1024]
    pool = [gen.batch(100 + k, B=1024) for k in range(2)]
    reps = 12
    singles = [workload.DeviceBatch(workload.slice_batch(pool[i % 2], cfg.T, 0, b)) for i, b in enumerate(grid)]
    order = [i for _ in range(reps) for i in range(len(grid))]
    lat = rec.serve_trace(model, [[singles[i]] for i in order], np.zeros(len(order)))
    step = np.diff(lat).reshape(-1)                      # step[j] = service time of request order[j + 1]
    per = {b: [] for b in grid}
    for j, dt in enumerate(step):
        if j + 1 >= len(grid):                           # the first pass warms caches and clocks up
            per[grid[order[j + 1]]].append(dt)
    tg = np.array([float(np.median(per[b])) for b in grid])
    table = np.zeros(1025)
    table[1:] = np.interp(np.arange(1, 1025), grid, tg)
    del singles

    cands = [1 << k for k in range(11)]
    res = {"service_us": {str(b): table[b] * 1e6 for b in (1, 16, 64, 256, 1024)}, "service_table_s": table.tolist(),
           "percentile": 0.95,
           "candidates": cands, "targets": {}}

    def tune(n_queries, targets):
        sizes = synth.lognormal_query_sizes(synth.MASTER_SEED, n_queries)
        unit = synth.unit_poisson_arrivals(synth.MASTER_SEED, n_queries)
        per_size = {B: np.array([rec.sched_query_service(n, B, table) for n in range(1001)]) for B in cands}
        svc = {B: per_size[B][sizes] for B in cands}
        for sla in targets:
            qps = [rec.sched_max_qps(unit, svc[B], 0.95, sla * 1e-3, 40) for B in cands]
            k = rec.sched_hill_climb(qps)
            res["targets"][f"{sla}ms"] = {"queries": n_queries, "max_qps": {str(B): q for B, q in zip(cands, qps)},
                                          "chosen_batch": cands[k], "chosen_max_qps": qps[k],
                                          "best_batch_exhaustive": cands[int(np.argmax(qps))]}
        return sizes, unit, svc

    # the paper's targets are seconds-scale against a ~0.1 ms service time: the trace must last many
    # times the target for the percentile to be a steady-state one, hence the longer trace
    medium = TABLE_II_TARGET_MS.get(cfg.name, 100.0)
    tune(100_000, [0.5 * medium, medium, 1.5 * medium])
    sizes, unit, svc = tune(synth.SWEEP_QUERIES, sla_ms)

    # live check at the second-loosest of the device-scale targets
    sla = sorted(sla_ms)[-2]
    pick = res["targets"][f"{sla}ms"]
    Bs, rate = pick["chosen_batch"], live_load * pick["chosen_max_qps"]
    if rate > 0:
        src = [gen.batch(100 + k, B=1000) for k in range(4)]
        staged = [[workload.DeviceBatch(workload.slice_batch(src[q % len(src)], cfg.T, s, c))
                   for s, c in rec.split_query(int(n), Bs)] for q, n in enumerate(sizes.tolist())]
        one = rec.ServeTrace(model, staged)
        one.run(np.zeros(len(staged)))                                           # warm
        live = one.run(unit / rate)
        want = rec.sched_fifo_latencies(unit / rate, svc[Bs])
        res["live"] = {"target_ms": sla, "batch": Bs, "offered_qps": rate, "load_vs_predicted_max": live_load,
                       "p95_ms": rec.sched_percentile(live, 0.95) * 1e3, "p50_ms": rec.sched_percentile(live, 0.5) * 1e3,
                       "predicted_p95_ms": rec.sched_percentile(want, 0.95) * 1e3,
                       "within_target": bool(rec.sched_percentile(live, 0.95) <= sla * 1e-3),
                       "items_per_s": float(sizes.sum() * rate / len(sizes))}
        # latency-bounded throughput measured, not modelled: the largest offered rate whose live
        # p95 stays under the target, one stream and the stream pool
        res["live_max_qps"] = {"target_ms": sla, "batch": Bs, "predicted_single_stream": pick["chosen_max_qps"],
                               "single_stream": live_max_qps(one, unit, sla * 1e-3, pick["chosen_max_qps"], rec)}
        if pool_streams is not None:
            many = rec.ServeTrace(model, staged, pool_streams)
            many.run(np.zeros(len(staged)))
            res["live_max_qps"][f"{len(pool_streams)}_streams"] = live_max_qps(many, unit, sla * 1e-3,
                                                                                pick["chosen_max_qps"], rec)
        del one, staged
        if pool_streams is not None:
            del many
    # the hill climb run the way the paper runs it: on measured rates, here with the stream pool
    if pool_streams is not None:
        res["live_hill_climb"] = {f"{t}ms": live_hill_climb(cfg, model, gen, sizes, unit, t * 1e-3, cands, pool_streams,
                                                            rec, workload, np) for t in (1.0, 5.0)}
        # the same with the requests of a query dealt over the streams (request-level parallelism)
        res["live_hill_climb_spread_requests"] = {
            f"{t}ms": live_hill_climb(cfg, model, gen, sizes, unit, t * 1e-3, cands, pool_streams, rec, workload, np,
                                      spread=True) for t in (0.25, 1.0)}
    return res


def cpu_request_table(cfg, gen, synth, workload, np, max_b=1024):
    """CPU-baseline leg: seconds for one request of b items on ONE host core, from the oracle run
    single-threaded on slices of a batch (b = 1, 2, 4, ..., linear in between)."""
    import oracle
    src = gen.batch(300, B=max_b)
    pb, pt = synth.mlp_params(cfg.bottom, 0), synth.mlp_params(cfg.top, 1)
    oracle.set_threads(1)
    grid, t = [], []
    b = 1
    while b <= max_b:
        part = workload.slice_batch(src, cfg.T, 0, b)
        tables, idx = synth.compact_tables(cfg.replace(B=b), part)
        best = 1e30
        for _ in range(3 if b <= 64 else 1):
            t0 = time.perf_counter()
            st, _ = oracle.model_forward(tables, pb.W, pb.b, pt.W, pt.b, part.dense, idx, part.lengths, bf16=cfg.bf16,
                                         concat=cfg.interaction == "concat")
            best = min(best, time.perf_counter() - t0)
            assert st == oracle.OK
        grid.append(b)
        t.append(best)
        b *= 2
    table = np.zeros(max_b + 1)
    table[1:] = np.interp(np.arange(1, max_b + 1), grid, t)
    return table


def offload_threshold_tuning(cfg, gpu_table, gen, torch, rec, synth, workload, np, n_queries=20_000):
    """Second hill climb of Section IV-C on the two-tier queueing model (Section IV-B): queries of
    tau items or more go to the device (service = measured request time + host-to-device copy of
    the query's inputs), the others are split into requests on the host's cores (request time =
    the oracle on one core: the only CPU implementation there is, a stand-in for a CPU serving
    path this library does not have).  Model only: no query is served on the CPU."""
    cores = min(16, os.cpu_count() or 1)
    c = cpu_request_table(cfg, gen, synth, workload, np)
    # host-to-device: one pinned copy of a full batch's inputs, and of a one-item batch
    big = gen.batch(301, B=1000)
    per_item = (big.dense.nbytes + big.indices.nbytes + big.lengths.nbytes) / 1000.0
    src = torch.empty(int(per_item * 1000), dtype=torch.uint8).pin_memory()
    dst = torch.empty_like(src, device="cuda")

    def copy_s(nbytes, reps=50):
        dst[:nbytes].copy_(src[:nbytes], non_blocking=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            dst[:nbytes].copy_(src[:nbytes], non_blocking=True)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps
    t_small, t_big = copy_s(int(per_item)), copy_s(int(per_item * 1000))
    m = np.arange(0, 1001)
    g = np.asarray(gpu_table)[:1001] + t_small + (t_big - t_small) * (m - 1) / 999.0
    g[0] = 0.0

    sizes = synth.lognormal_query_sizes(synth.MASTER_SEED, n_queries)
    unit = synth.unit_poisson_arrivals(synth.MASTER_SEED, n_queries)
    medium = TABLE_II_TARGET_MS.get(cfg.name, 100.0)
    res = {"cpu_workers": cores, "queries": n_queries,
           "cpu_request_ms": {str(b): c[b] * 1e3 for b in (1, 16, 64, 256, 1024)},
           "device_query_ms_with_copy": {str(b): g[b] * 1e3 for b in (1, 16, 64, 256, 1000)}, "targets": {}}
    batches = [1 << i for i in range(11)]
    taus = [1 << i for i in range(11)] + [1001]                    # 1001: nothing goes to the device
    for sla in (0.5 * medium, medium):
        s = sla * 1e-3
        # first climb: request batch size for the CPU tier alone
        cpu_qps = []
        for B in batches:
            cpu_qps.append(rec.sched_two_tier_max_qps(unit, sizes, 1001, B, c, cores, g, 0.95, s, 30))
            if len(cpu_qps) > 1 and cpu_qps[-1] < cpu_qps[-2]:
                break
        kb = rec.sched_hill_climb(cpu_qps)
        B = batches[kb]
        # second climb: query-size threshold, from "everything on the device" upwards
        qps = []
        for tau in taus:
            qps.append(rec.sched_two_tier_max_qps(unit, sizes, tau, B, c, cores, g, 0.95, s, 30))
            if len(qps) > 1 and qps[-1] < qps[-2]:
                break
        kt = rec.sched_hill_climb(qps)
        res["targets"][f"{sla:g}ms"] = {"cpu_batch": B, "cpu_only_max_qps": {str(b): q for b, q in zip(batches, cpu_qps)},
                                        "max_qps_by_threshold": {str(t): q for t, q in zip(taus, qps)},
                                        "chosen_threshold": taus[kt], "chosen_max_qps": qps[kt]}
        print(f"[sched] threshold climb, target {sla:g} ms: cpu batch {B}, threshold {taus[kt]}, {qps[kt]:.0f} queries/s",
              file=sys.stderr, flush=True)
    return res


def live_hill_climb(cfg, model, gen, sizes, unit, sla_s, cands, pool_streams, rec, workload, np, n=400, spread=False):
    """Section IV-C on live measurements: for batch sizes 1, 2, 4, ... measure the largest Poisson
    rate the device sustains with p95 <= target (first `n` queries of the trace, requests spread
    over the stream pool) and climb until that rate degrades."""
    src = [gen.batch(100 + k, B=1000) for k in range(4)]
    qps = []
    for Bs in cands:
        staged = [[workload.DeviceBatch(workload.slice_batch(src[q % len(src)], cfg.T, s, c))
                   for s, c in rec.split_query(int(m), Bs)] for q, m in enumerate(sizes[:n].tolist())]
        tr = rec.ServeTrace(model, staged, pool_streams, spread_requests=spread)
        tr.run(np.zeros(n))                                               # warm
        idle = tr.run(np.arange(n) * 2.0 * sla_s)                         # no queueing: service times alone
        if rec.sched_percentile(idle, 0.95) > sla_s:
            qps.append(0.0)
        else:
            start = max(qps[-1] if qps else 0.0, 0.5 / sla_s)
            qps.append(live_max_qps(tr, unit[:n], sla_s, start, rec, bracket_steps=14, bisect_steps=4))
        del tr, staged
        print(f"[sched] live climb{' (requests spread)' if spread else ''}, target {sla_s * 1e3:g} ms, batch {Bs}: "
              f"{qps[-1]:.0f} queries/s", file=sys.stderr, flush=True)
        if len(qps) > 1 and qps[-1] < qps[-2]:
            break                                                          # degraded: the climb stops here
    k = rec.sched_hill_climb(qps)
    return {"queries": n, "max_qps": {str(B): q for B, q in zip(cands, qps)}, "chosen_batch": cands[k],
            "chosen_max_qps": qps[k]}


def live_max_qps(trace, unit, sla_s, start, rec, grow=1.25, bracket_steps=10, bisect_steps=6):
    """Largest offered rate (queries/s) for which a live replay keeps p95 <= sla_s: bracket from
    `start` by factors of `grow`, then bisect.  Each probe replays the whole trace once."""
    ok = lambda r: rec.sched_percentile(trace.run(unit / r), 0.95) <= sla_s
    lo = hi = None
    r = start
    if ok(r):
        lo = r
        for _ in range(bracket_steps):
            r *= grow
            if ok(r):
                lo = r
            else:
                hi = r
                break
    else:
        hi = r
        for _ in range(bracket_steps):
            r /= grow
            if ok(r):
                lo = r
                break
            hi = r
    if lo is None:
        return 0.0
    if hi is None:
        return lo
    for _ in range(bisect_steps):
        mid = 0.5 * (lo + hi)
        if ok(mid):
            lo = mid
        else:
            hi = mid
    return lo


if __name__ == "__main__":
    main()
