#!/usr/bin/env python3
"""Benchmark of the AET-SGD hot path on one MI355X.

A "step" is one whole job of the workload: every client's local rounds (threshold
s_i = a*i + b, all rounds), every server aggregation under the delay schedule, until the
message queue has drained.  Inputs (shards, initial model) are resident in HBM before the
timed region; the timed region holds K jobs, each restarted with aet_reset.

Prints ONE JSON line with the throughput in client-samples/s, the roofline record of the
dominant kernel (its launches are timed live with HIP events on the library's stream),
and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth
FP32_MFMA_PEAK_TFLOPS = 157.3   # MI355X published dense fp32 matrix rate


def per_step_bytes(model, fam_name):
    """Algorithmic bytes one client moves in one SGD recursion inside the kernels of one
    family (replicas and U live in HBM and are touched every recursion)."""
    import workloads as W
    B = model.batch
    shp = model.shapes()
    D = model.in_size()
    P = model.n_params()
    total = 0
    if fam_name == "k_mlp_round":
        # streaming model: read+write W, read+write U, the mini-batch rows and labels
        return 16 * P + B * (4 * D + 4)
    if fam_name == "k_softmax_round":
        # compulsory model (replica and U stay on chip for the round): rows and labels;
        # the 12 P bytes per round for reading w_global and writing w_c and U are added
        # by the caller
        return B * (4 * D + 4)
    if fam_name == "k_gather":
        return B * (8 * D + 8)
    if fam_name == "k_softmax_ce":
        return B * (8 * model.n_classes() + 4)
    for L, sl, (c, h, w), (oc, oh, ow) in zip(model.layers, model.param_slices(), shp[:-1], shp[1:]):
        n_in, n_out = c * h * w, oc * oh * ow
        if L.type == W.DENSE:
            nw = sl[1] + sl[3]
            if fam_name == "k_dense_fwd":
                total += 4 * nw + 4 * B * (n_in + n_out)
            elif fam_name == "k_dense_bwd_data":
                total += 4 * sl[1] + 4 * B * (n_in + n_out)
            elif fam_name == "k_dense_bwd_weight":
                total += 16 * nw + 4 * B * (n_in + n_out)
        elif L.type == W.CONV:
            nw = sl[1] + sl[3]
            if fam_name == "k_conv_fwd":
                total += 4 * nw + 4 * B * (n_in + n_out)
            elif fam_name == "k_conv_bwd_data":
                total += 4 * sl[1] + 4 * B * (n_in + n_out)
            elif fam_name == "k_conv_bwd_weight":
                total += 16 * nw + 4 * B * (n_in + n_out)
        else:
            if fam_name == "k_pool_fwd":
                total += B * (4 * n_in + 5 * n_out)
            elif fam_name == "k_pool_bwd":
                total += B * (4 * n_in + 5 * n_out)
    return total


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
    src = {"k_mlp_round": "kernels_mlp.hip", "k_softmax_round": "kernels_softmax.hip"}.get(fam_name)
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


def per_step_flops(model, fam_name):
    """Useful flops (2 per multiply-add, no tile padding) one client spends in one SGD
    recursion inside the matrix-core kernels of one family; 0 for the other families."""
    import workloads as W
    B = model.batch
    shp = model.shapes()
    total = 0
    first = True
    for L, sl, (c, h, w), (oc, oh, ow) in zip(model.layers, model.param_slices(), shp[:-1], shp[1:]):
        if L.type == W.DENSE:
            macs = B * sl[1]
            kind = "dense"
        elif L.type == W.CONV:
            macs = B * sl[1] * oh * ow
            kind = "conv"
        else:
            continue
        if fam_name == f"k_{kind}_fwd" or fam_name == f"k_{kind}_bwd_weight":
            total += 2 * macs
        elif fam_name == f"k_{kind}_bwd_data" and not first:   # no dX for the first layer
            total += 2 * macs
        first = False
    return total


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


def cpu_baseline(wl, budget_s=12.0):
    """The fp64 oracle as it stands, on the host cores, for about budget_s seconds of the
    same workload from its start (whole ticks; a workload that finishes earlier is started
    again from scratch); client-samples per second."""
    from oracle import Oracle
    threads = min(wl.n_clients, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    done = ticks = passes = 0
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < budget_s:
        orc = Oracle(wl, "f64")
        passes += 1
        while not orc.all_done() and time.perf_counter() - t0 < budget_s:
            for c, k in orc.run_round():
                done += orc.round_info(c, k)["s"]
            orc.exchange()
            ticks += 1
        orc.close()
    dt = time.perf_counter() - t0
    return dict(value=done / dt, unit="client-samples/s", cores=threads, kind="oracle",
                sample=f"{ticks} ticks of the same workload from its start, {passes} pass(es) "
                       f"({done} client-samples, {dt:.1f} s, fp64, one thread per client)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (default 2: the MLP)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rounds", type=int, default=0, help="exploration only: fewer rounds per client")
    ap.add_argument("--topology", choices=["server", "ring"], default="server",
                    help="server: clients and a server (default); ring: peer-to-peer form, every "
                         "node sends to its two ring neighbours")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (calibrates the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as W
    from paper_2112_13935_amd.runner import Run

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    wl = W.CONFIGS[args.config]()
    if args.rounds > 0:
        wl.rounds = args.rounds
        wl.name += f"_first{args.rounds}rounds"
    if args.topology == "ring":
        wl.topology = W.ring_topology(wl.n_clients)
        wl.agg_scale = 1.0 / 3.0      # a node and its two neighbours
        wl.name += "_ring"
    run = Run(wl)
    names = run.lib.profile_family_names()
    total_samples = wl.total_client_samples()
    total_steps = wl.n_clients * sum((wl.a * i + wl.b) // wl.model.batch for i in range(wl.rounds))

    def job():
        run.lib.aet_reset()
        return run.run_ticks()

    for _ in range(max(args.warmup, 0)):
        job()
    run.lib.aet_synchronize()

    if args.copy_probe:
        # a plain copy of known size: reads 256 MiB and writes 256 MiB per dispatch
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # which kernel family dominates: one untimed job with every family's launches timed
    run.lib.aet_profile_enable(-1, True)
    job()
    fam_ms = [run.lib.aet_profile_read(f) for f in range(len(names))]
    run.lib.aet_profile_enable(-1, False)
    dom = int(np.argmax([ms for _, ms in fam_ms]))
    total_ms = max(sum(ms for _, ms in fam_ms), 1e-12)
    share = fam_ms[dom][1] / total_ms
    shares = {names[f]: round(ms / total_ms, 4) for f, (_, ms) in enumerate(fam_ms) if ms > 0}

    run.lib.aet_profile_enable(dom, True)
    run.lib.aet_synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ticks = 0
    for _ in range(args.steps):
        ticks = job()
    run.lib.aet_synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    launches, kernel_ms = run.lib.aet_profile_read(dom)
    run.lib.aet_profile_enable(dom, False)

    ms_per_step = dt * 1e3 / args.steps
    value = total_samples * args.steps / dt
    fam = names[dom]
    bytes_per_job = per_step_bytes(wl.model, fam) * total_steps
    model_name = "streaming (16P + B(4D+4) per recursion)"
    if fam == "k_softmax_round":
        bytes_per_job += 12 * wl.model.n_params() * wl.n_clients * wl.rounds
        model_name = "compulsory (B(4D+4) per recursion + 12P per round)"
    elif fam != "k_mlp_round":
        model_name = "per-kernel operand bytes"
    launches_per_job = launches / args.steps
    avg_launch_ms = kernel_ms / max(launches, 1)
    achieved = (bytes_per_job / launches_per_job) / (avg_launch_ms * 1e-3) / 1e9
    roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": fam, "byte_model": model_name,
            "avg_launch_us": avg_launch_ms * 1e3, "launches_per_step": launches_per_job,
            "algorithmic_bytes_per_launch": bytes_per_job / launches_per_job}
    flops_per_job = per_step_flops(wl.model, fam) * total_steps
    if flops_per_job > 0:
        # a contraction on the matrix cores: priced against the fp32 MFMA peak
        tf = (flops_per_job / launches_per_job) / (avg_launch_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": tf, "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / FP32_MFMA_PEAK_TFLOPS, "traffic": None, "kernel": fam,
                "flop_model": "useful multiply-adds x 2, no tile padding",
                "avg_launch_us": avg_launch_ms * 1e3, "launches_per_step": launches_per_job,
                "algorithmic_flops_per_launch": flops_per_job / launches_per_job}
    if args.rounds == 0 and args.topology == "server":
        roof["traffic"] = counter_traffic(fam, wl.name)
    roof["share_of_kernel_time"] = share
    roof["kernel_time_shares"] = shares
    recv = receive_record(run, wl, names)
    out = {
        "metric": "client SGD samples/sec (all clients, 1 GPU)",
        "value": value, "unit": "client-samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "n_clients": wl.n_clients, "rounds": wl.rounds,
                   "batch": wl.model.batch, "threshold": f"s_i = {wl.a}*i + {wl.b}",
                   "client_samples_per_step": total_samples, "ticks_per_step": ticks,
                   "params": wl.model.n_params(), "agg_scale": wl.agg_scale},
        "roofline": roof,
    }
    out["config"]["topology"] = args.topology
    if recv is not None:
        out["receive"] = recv
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    run.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
