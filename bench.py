#!/usr/bin/env python3
"""Benchmark of the AET-SGD hot path on one MI355X.

A "step" is one whole job of a workload: every client's local rounds (threshold
s_i = a*i + b, all rounds), every server aggregation under the delay schedule, until the
message queue has drained.  Inputs (shards, initial model) are resident in HBM before the
timed region; the timed region holds K jobs, each restarted with aet_reset.

All five workloads are timed in one run.  The headline (`value`, `config`, `roofline`,
`cpu_baseline`) is the largest one, the 1,024-client softmax-3072 workload; the other four
are reported under `configs` with the same fields.  --config k times workload k alone (it
becomes the headline).

Per workload: throughput in client-samples/s; the dominant kernel family (found by one
untimed job with every family's launches bracketed by HIP events on the library's stream),
its launches timed the same way inside the timed region; the roofline record of that
kernel; the tick's second half (server reduce) timed over one more job; and the CPU
oracle on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
FP32_MFMA_PEAK_TFLOPS = 157.3    # MI355X published dense fp32 matrix rate
FP32_VECTOR_PEAK_TFLOPS = 157.3  # published fp32 vector rate (two flops per lane and clock
#                                  need the packed forms; single-issue FMA code tops out at 78.6)
HEADLINE = 5
FUSED = ("k_softmax_round", "k_mlp_round", "k_lenet_round")


def layer_macs(model):
    """Per sample and parameter layer: (kind, multiply-adds of the forward product,
    is it the first parameter layer)."""
    import workloads as W
    shp = model.shapes()
    out, first = [], True
    for L, sl, (oc, oh, ow) in zip(model.layers, model.param_slices(), shp[1:]):
        if L.type == W.DENSE:
            out.append(("dense", sl[1], first))
        elif L.type == W.CONV:
            out.append(("conv", sl[1] * oh * ow, first))
        else:
            continue
        first = False
    return out


def recursion_flops(model):
    """Useful flops of one SGD recursion of one client: forward, backward-weight, backward-data
    (none for the first layer), 2 flops per multiply-add, no tile padding, plus 3 per
    parameter for  w <- w - eta g,  U <- U + g."""
    macs = sum(m * (2 if first else 3) for _, m, first in layer_macs(model))
    return 2 * model.batch * macs + 3 * model.n_params()


def family_flops(model, fam_name):
    """... of which inside the matrix-core kernels of one layer-engine family."""
    total = 0
    for kind, m, first in layer_macs(model):
        if fam_name in (f"k_{kind}_fwd", f"k_{kind}_bwd_weight"):
            total += 2 * model.batch * m
        elif fam_name == f"k_{kind}_bwd_data" and not first:
            total += 2 * model.batch * m
    return total


def byte_models(model, recursions, client_rounds):
    """The two byte models of a whole job.
    compulsory: what has to move when a replica stays on chip for its round: the sampled
    rows and labels of every recursion, and per round one read of the global model and one
    write each of w_c and U.
    streaming: replica and U live in HBM and are read and written in every recursion."""
    B, D, P = model.batch, model.in_size(), model.n_params()
    rows = B * (4 * D + 4)
    return {"compulsory": rows * recursions + 12 * P * client_rounds,
            "streaming": (16 * P + rows) * recursions}


def counter_traffic(fam_name, workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter
    summary (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a
    plain copy of known size), or None: no summary for this kernel and workload, or the
    kernel source has changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"{fam_name}_{workload}_pmc.md")
    if not os.path.exists(path):
        return None
    rec = {}
    for line in open(path):
        parts = line.strip().split(": ", 1)
        if len(parts) == 2 and line.startswith("    "):
            rec[parts[0]] = parts[1]
    src = {"k_mlp_round": "kernels_mlp.hip", "k_softmax_round": "kernels_softmax.hip",
           "k_lenet_round": "kernels_lenet.hip"}.get(fam_name)
    if src is None or "source_sha256" not in rec:
        return None
    h = hashlib.sha256()
    for f in (src, "aet_device.h", "aet_internal.h"):
        with open(os.path.join(ROOT, "paper_2112_13935_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    if h.hexdigest() != rec["source_sha256"]:
        return None
    try:
        return 1024.0 * (float(rec["fetch_kib_per_launch"]) * float(rec["fetch_scale"]) +
                         float(rec["write_kib_per_launch"]) * float(rec["write_scale"]))
    except (KeyError, ValueError):
        return None


def receive_record(run, wl, names):
    """The tick's second half (server reduce, or Receive at the neighbours) timed over one
    job run tick by tick: algorithmic bytes = read+write of every model that changes (8P)
    plus one read of every U per model it is applied to (4P)."""
    fam = names.index("k_apply_neighbour_U" if run.p2p else "server_reduce")
    P4 = 4 * wl.model.n_params()
    run.lib.aet_reset()
    run.lib.aet_profile_enable(fam, True)
    nbytes = 0
    if run.p2p:
        off, nbr = wl.topology
    while not run.lib.aet_all_done(wl.rounds):
        run.run_round()
        senders = [c for c, _ in run.exchange()]
        if not senders:
            continue
        if run.p2p:
            receivers = set()
            for c in senders:
                receivers.update(nbr[off[c]:off[c + 1]].tolist())
            nbytes += 2 * P4 * len(receivers) + P4 * sum(int(off[c + 1] - off[c]) for c in senders)
        else:
            nbytes += 2 * P4 + P4 * len(senders)
    launches, ms = run.lib.aet_profile_read(fam)
    run.lib.aet_profile_enable(fam, False)
    if launches == 0 or ms <= 0:
        return None
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"kernel": names[fam], "bound": "hbm", "launches_per_step": launches,
            "avg_launch_us": ms * 1e3 / launches, "algorithmic_bytes_per_launch": nbytes / launches,
            "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}


def oracle_leg(wl, n_clients, budget_s):
    """The fp64 oracle as it stands for about budget_s seconds of the workload from its
    start, restricted to the first n_clients clients (one thread per client; one client =
    one thread); whole ticks, at least one.  A workload that finishes earlier is started
    again from scratch."""
    from oracle import Oracle
    done = ticks = passes = 0
    t0 = time.perf_counter()
    while ticks == 0 or time.perf_counter() - t0 < budget_s:
        orc = Oracle(wl, "f64", n_clients=n_clients)
        passes += 1
        while not orc.all_done() and (ticks == 0 or time.perf_counter() - t0 < budget_s):
            for c, k in orc.run_round():
                done += orc.round_info(c, k)["s"]
            orc.exchange()
            ticks += 1
        orc.close()
    dt = time.perf_counter() - t0
    return done / dt, (f"{ticks} ticks from the workload's start, first {n_clients} of {wl.n_clients} clients, "
                       f"{passes} pass(es): {done} client-samples in {dt:.1f} s")


def cpu_baseline(wl, budget_s, single_thread):
    threads = min(wl.n_clients, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    v, sample = oracle_leg(wl, threads, budget_s)
    out = dict(value=v, unit="client-samples/s", cores=threads, kind="oracle", precision="fp64",
               sample=sample + "; one thread per client")
    if single_thread:
        v1, s1 = oracle_leg(wl, 1, budget_s)
        out["single_thread"] = dict(value=v1, unit="client-samples/s", cores=1, precision="fp64", sample=s1)
    return out


def measure(cfg, steps, warmup, args, headline):
    """Times one workload; returns its record."""
    import torch
    import workloads as W
    from paper_2112_13935_amd.runner import Run

    wl = W.CONFIGS[cfg]()
    if args.rounds > 0:
        wl.rounds = args.rounds
        wl.name += f"_first{args.rounds}rounds"
    if args.topology == "ring":
        wl.topology = W.ring_topology(wl.n_clients)
        wl.agg_scale = 1.0 / 3.0      # a node and its two neighbours
        wl.name += "_ring"
    run = Run(wl)
    names = run.lib.profile_family_names()
    model = wl.model
    total_samples = wl.total_client_samples()
    recursions = wl.n_clients * sum((wl.a * i + wl.b) // model.batch for i in range(wl.rounds))
    client_rounds = wl.n_clients * wl.rounds

    def job():
        run.lib.aet_reset()
        return run.run_ticks()

    for _ in range(max(warmup, 0)):
        job()
    run.lib.aet_synchronize()

    # which kernel family dominates: one untimed job with every family's launches timed
    run.lib.aet_profile_enable(-1, True)
    job()
    fam_ms = [run.lib.aet_profile_read(f) for f in range(len(names))]
    run.lib.aet_profile_enable(-1, False)
    dom = int(np.argmax([ms for _, ms in fam_ms]))
    total_ms = max(sum(ms for _, ms in fam_ms), 1e-12)
    shares = {names[f]: round(ms / total_ms, 4) for f, (_, ms) in enumerate(fam_ms) if ms > 0}
    launches_all = sum(n for n, _ in fam_ms)

    run.lib.aet_profile_enable(dom, True)
    run.lib.aet_synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ticks = 0
    for _ in range(steps):
        ticks = job()
    run.lib.aet_synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    launches, kernel_ms = run.lib.aet_profile_read(dom)
    run.lib.aet_profile_enable(dom, False)

    fam = names[dom]
    value = total_samples * steps / dt
    launches_per_job = launches / steps
    avg_launch_s = kernel_ms * 1e-3 / max(launches, 1)
    kernel_s_per_job = kernel_ms * 1e-3 / steps
    bm = byte_models(model, recursions, client_rounds)
    job_flops = recursion_flops(model) * recursions
    fused = fam in FUSED

    def hbm(nbytes, label):
        a = nbytes / kernel_s_per_job / 1e9
        return {"model": label, "achieved": a, "unit": "GB/s", "frac": a / HBM_PEAK_GBS,
                "bytes_per_launch": nbytes / launches_per_job}

    def flops(nflops, peak):
        a = nflops / kernel_s_per_job / 1e12
        return {"achieved": a, "unit": "TFLOP/s", "peak": peak, "frac": a / peak,
                "flops_per_launch": nflops / launches_per_job,
                "flop_model": "useful multiply-adds x 2, no tile padding (+ 3 per parameter and recursion for the update)"}

    traffic = counter_traffic(fam, wl.name) if (args.rounds == 0 and args.topology == "server") else None
    if fam == "k_softmax_round":
        # one dense layer, B = 1: rank-1 work on the vector ALU; the kernel keeps replica and U
        # on chip, so what it has to move is the compulsory model
        c = hbm(bm["compulsory"], "compulsory: B(4D+4) per recursion + 12P per round (replica on chip)")
        roof = {"bound": "hbm", "achieved": c["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": c["frac"],
                "traffic": traffic, "byte_model": c["model"], "algorithmic_bytes_per_launch": c["bytes_per_launch"],
                "streaming_equivalent": hbm(bm["streaming"], "streaming: 16P + B(4D+4) per recursion (bytes the kernel does not move)"),
                "alu": flops(job_flops, FP32_VECTOR_PEAK_TFLOPS)}
    elif fused:
        # contractions on the matrix cores with the replica on chip
        f = flops(job_flops, FP32_MFMA_PEAK_TFLOPS)
        roof = {"bound": "mfma", "achieved": f["achieved"], "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": f["frac"], "traffic": traffic, "flop_model": f["flop_model"],
                "algorithmic_flops_per_launch": f["flops_per_launch"],
                "hbm_compulsory": hbm(bm["compulsory"], "compulsory: B(4D+4) per recursion + 12P per round (replica on chip)"),
                "hbm_streaming_equivalent": hbm(bm["streaming"], "streaming: 16P + B(4D+4) per recursion (bytes the kernel does not move)")}
    else:
        # a layer-engine family: its own useful flops against the fp32 matrix peak
        ff = family_flops(model, fam) * recursions
        f = flops(ff, FP32_MFMA_PEAK_TFLOPS) if ff > 0 else None
        if f is not None:
            roof = {"bound": "mfma", "achieved": f["achieved"], "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": f["frac"], "traffic": None, "flop_model": "useful multiply-adds x 2, no tile padding",
                    "algorithmic_flops_per_launch": f["flops_per_launch"]}
        else:
            c = hbm(bm["streaming"] * kernel_ms / max(total_ms, 1e-12), "streaming, this family's share")
            roof = {"bound": "hbm", "achieved": c["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": c["frac"], "traffic": None, "byte_model": c["model"]}
    roof.update({"kernel": fam, "avg_launch_us": avg_launch_s * 1e6, "launches_per_step": launches_per_job,
                 "share_of_kernel_time": fam_ms[dom][1] / total_ms, "kernel_time_shares": shares,
                 "launches_per_step_all_families": launches_all})
    # the whole job against the wall clock (launch gaps, server step and host included)
    wall = dt / steps
    roof["whole_job"] = {
        "useful_tflops": job_flops / wall / 1e12,
        "frac_of_fp32_mfma_peak": job_flops / wall / 1e12 / FP32_MFMA_PEAK_TFLOPS,
        "compulsory_gbs": bm["compulsory"] / wall / 1e9,
        "frac_of_hbm_peak_compulsory": bm["compulsory"] / wall / 1e9 / HBM_PEAK_GBS,
        "streaming_equivalent_gbs": bm["streaming"] / wall / 1e9,
        "frac_of_hbm_peak_streaming_equivalent": bm["streaming"] / wall / 1e9 / HBM_PEAK_GBS}
    recv = receive_record(run, wl, names)
    out = {
        "value": value, "unit": "client-samples/s", "steps": steps, "warmup": warmup,
        "ms_per_step": dt * 1e3 / steps, "timed_region_s": dt,
        "config": {"workload": wl.name, "n_clients": wl.n_clients, "rounds": wl.rounds,
                   "batch": model.batch, "threshold": f"s_i = {wl.a}*i + {wl.b}",
                   "client_samples_per_step": total_samples, "ticks_per_step": ticks,
                   "params": model.n_params(), "agg_scale": wl.agg_scale, "topology": args.topology},
        "roofline": roof,
    }
    if recv is not None:
        out["receive"] = recv
    run.close()
    del run
    gc.collect()
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, 10.0 if headline else 3.0, single_thread=headline)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=0,
                    help="0 (default): all five workloads, the 1,024-client one as the headline; k: workload k alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rounds", type=int, default=0, help="exploration only: fewer rounds per client")
    ap.add_argument("--topology", choices=["server", "ring"], default="server",
                    help="server: clients and a server (default); ring: peer-to-peer form, every "
                         "node sends to its two ring neighbours")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (calibrates the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1 (there is no multi-GPU path)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    if args.copy_probe:
        # a plain copy of known size: reads 256 MiB and writes 256 MiB per dispatch
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head_cfg = args.config if args.config else HEADLINE
    head = measure(head_cfg, args.steps, args.warmup, args, headline=True)
    out = {"metric": "client SGD samples/sec (all clients, 1 GPU)", "value": head["value"],
           "unit": head["unit"], "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic", "config": head["config"],
           "timed_region_s": head["timed_region_s"], "roofline": head["roofline"]}
    for k in ("receive", "cpu_baseline"):
        if k in head:
            out[k] = head[k]
    if not args.config:
        # the other four workloads; the CNN job takes seconds, so it gets fewer steps
        out["configs"] = {}
        for cfg in (1, 2, 3, 4):
            steps = max(1, args.steps // 5) if cfg == 4 else args.steps
            rec = measure(cfg, steps, min(args.warmup, 1), args, headline=False)
            out["configs"][rec["config"]["workload"]] = rec
        out["timed_region_s_all_workloads"] = head["timed_region_s"] + sum(
            r["timed_region_s"] for r in out["configs"].values())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
