#!/usr/bin/env python3
"""Benchmark of the error-feedback AMSGrad step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config IDX]

With no --config it runs the largest of the five workloads (cfg4: n = 8 workers, d = 110 M coordinates,
Top-k with k = 110 000; every array streams from HBM); the other four are behind --config 0..3.

One "step" is one pass of the whole hot path (error-feedback add, compression, error update,
average over the n simulated workers, AMSGrad update) over one batch of synthetic gradients that
is already resident in HBM.  Prints ONE JSON line:
  value        coordinates/s = n*d / step time over K timed steps (profiling off)
  roofline     the dominant kernel's algorithmic bytes / its average duration measured with HIP
               events on the step's stream (a second run of K steps with per-kernel events on)
  cpu_baseline the CPU oracle timed on this machine's host cores on a bounded number of steps
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak

PROFILES = os.path.join(ROOT, "profiles")
CSRC = os.path.join(ROOT, "paper_2111_00705_amd", "csrc")

# rocprofv3 summaries under profiles/ exist per workload and variant of the run; a variant's file name suffix:
PROFILE_SUFFIX = {"ef": "", "cd": "_cd_adam", "naive": "_naive", "none": "_uncompressed", "bf16": "_bf16",
                  "randk": "_randk"}

# The templated kernel behind each timing slot, by variant: which row of a rocprofv3 summary a slot reads.
KERNEL_VARIANT = {
    ("tk_pass1", "ef"): "cams::tk_pass1<0, float>", ("tk_pass1", "cd"): "cams::tk_pass1<1, float>",
    ("tk_pass1", "naive"): "cams::tk_pass1<3, float>", ("tk_pass1", "randk"): "cams::tk_pass1<0, float>",
    ("tk_pass1", "bf16"): "cams::tk_pass1<0, unsigned short>",
    ("bs_pass_update", "ef"): "cams::bs_pass_update<true, float",      # the steady-state variant (stored rows pending)
}


def run_variant(method: str, grad_dtype: str, randk: bool):
    """Which profiles/ summary a run corresponds to (None: there is none for this combination)."""
    if grad_dtype == "bf16" and method == "ef" and not randk:
        return "bf16"
    if grad_dtype != "f32":
        return None
    if randk:
        return "randk" if method == "ef" else None
    return method


def library_fingerprint() -> str:
    """Twelve hex digits of a SHA-1 over the library's sources (csrc/*, comments and white space removed): every rocprofv3 summary under
    profiles/ records the fingerprint of the build it was taken with, and counter figures are quoted from
    a summary only while it matches the sources in the tree."""
    import hashlib
    import re
    h = hashlib.sha1()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".h", ".hip")):
            text = open(os.path.join(CSRC, name), encoding="utf-8").read()
            # comments and layout do not change what is compiled: they are left out of the fingerprint
            text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
            text = re.sub(r"//[^\n]*", " ", text)
            h.update(name.encode())
            h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:12]


def measured_traffic(workload: str, variant, slot: str):
    """HBM-side bytes per launch (fetched + written) of one kernel from the rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE summary of this workload and variant (see run_variant) under profiles/ (a separate run,
    calibrated on probe_copy).
    Returns (bytes or None, source or reason).  None when there is no summary for this workload and
    variant, when it was taken with other sources than the tree holds, or when it has no row for the
    kernel variant that ran."""
    if variant is None:
        return None, "no counter summary for this method / gradient type"
    rel = os.path.join("profiles", workload + PROFILE_SUFFIX[variant] + ".md")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, f"{rel} does not exist"
    text = open(path).read()
    import re
    fp = re.search(r"Library source fingerprint: `([0-9a-f]{12})`", text)
    have = library_fingerprint()
    if not fp or fp.group(1) != have:
        return None, f"{rel} was taken with sources {fp.group(1) if fp else 'unrecorded'}, the tree holds {have}"
    want = KERNEL_VARIANT.get((slot, variant), "cams::" + slot)
    section = text.split("## HBM-side traffic", 1)[-1]
    for line in section.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        name = cells[0].strip("`")
        if len(cells) == 7 and (name == want or name.startswith(want + "<") or ("<" in want and name.startswith(want))):
            return float(cells[6]) * 1e6, rel
    return None, f"{rel} has no row for {want}"


def kernel_algorithmic_bytes(name: str, n: int, d: int, method: str = "ef") -> int:
    """Algorithmic bytes of one launch = per-unit figure x units (n*d worker-coordinates).
    The streaming pass of either compressor carries the 12 B per (worker, coordinate) of the
    method (read g, read the stored error / Markov vector, write it back); the update kernel carries
    the 32 B per coordinate of optimiser state (read and write theta, m, v, vhat).  CD-Adam's server
    stage reads and writes ghat and reads gtilde (12 B per coordinate); its last kernel reads and
    writes gtilde and the optimiser state (40 B per coordinate)."""
    nd = n * d
    naive = method == "naive"         # naive compression reads g only
    return {
        "bs_pass": (4 if naive else 12) * nd,
        # one launch: the pass of this step and the deferred update of the step before
        "bs_pass_update": 12 * nd + 32 * d,
        "bs_update": 32 * d,
        # CD-Adam with Top-k only reads g and ghat_i in the pass (ghat_i changes on the k kept coordinates)
        "tk_pass1": (4 if naive else 8 if method == "cd" else 12) * nd,
        "tk_final": 32 * d,
        "bs_server": 12 * d,
        "bs_apply": 40 * d,
        "tk_merge": 8 * d,
        "tk_pass1_server": 8 * d,
        "tk_apply": 40 * d,
        "plain_update": 4 * nd + 32 * d,
    }.get(name, 0)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: 200 on the three large workloads - under half a second of timed work "
                         "on the largest - and 1000 on the two small ones)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4,
                    help="index into the five named workloads; the default, 4, is the largest (n = 8, d = 110 M, Top-k: "
                         "14.08 GB of algorithmic traffic per step, far beyond every cache)")
    ap.add_argument("--buffers", type=int, default=None,
                    help="distinct gradient batches cycled through (default: 2 on the two largest workloads, "
                         "3.3 - 3.5 GB each, else 4)")
    ap.add_argument("--fingerprint", action="store_true", help="print the library source fingerprint and exit")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="budget of the oracle timing leg")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--method", choices=("ef", "cd", "naive", "none"), default="ef",
                    help="ef: error feedback (the headline metric); cd: CD-Adam, Algorithm 1; naive: compression "
                         "without memory; none: no compression")
    ap.add_argument("--grad-dtype", choices=("f32", "bf16", "f16"), default="f32",
                    help="f32: comp_ams_step (the headline metric); bf16 / f16: comp_ams_step_bf16 / _f16 on the "
                         "gradients rounded to that type (2 instead of 4 bytes read per gradient element)")
    ap.add_argument("--randk", action="store_true",
                    help="on a Top-k workload: Rand-k (Appendix A) with the same k instead of Top-k")
    ap.add_argument("--probe-mib", type=int, default=1024,
                    help="size of the plain-copy probe (MiB per buffer); 0 skips the copy ceiling")
    args = ap.parse_args()
    if args.fingerprint:
        print(library_fingerprint())
        return 0
    if args.steps is None:
        args.steps = 200 if args.config >= 2 else 1000
    if args.buffers is None:
        args.buffers = 2 if args.config >= 3 else 4
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all n workers are simulated as a batch on it); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2111_00705_amd as P
    import workloads as W

    w = W.get(args.config)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream().cuda_stream

    scales = w.scales()
    nbuf = max(1, min(args.buffers, args.steps))
    host_grads = [w.grads(t, scales=scales) for t in range(nbuf)]
    bf16 = args.grad_dtype != "f32"           # either 16-bit type
    if bf16:
        narrow = torch.bfloat16 if args.grad_dtype == "bf16" else torch.float16
        dev_grads = [torch.from_numpy(g).to(narrow).cuda() for g in host_grads]
        host_grads = [g.float().cpu().numpy() for g in dev_grads]      # what the oracle leg sees: the widened values
    else:
        dev_grads = [torch.from_numpy(g).cuda() for g in host_grads]

    kb = w.k if w.compressor == W.TOPK else (w.block if w.block else w.d)
    if args.randk and w.compressor != W.TOPK:
        print("bench.py: --randk needs a Top-k workload (--config 0, 2 or 4)", file=sys.stderr)
        return 2
    compressor = P.RANDK if args.randk else w.compressor          # the oracle uses the same numbers
    h = P.CompAms(w.d, w.n, compressor, kb, w.beta1, w.beta2, w.eps, w.lr)
    if w.compressor == W.BLOCKSIGN and w.layer_blocks:
        h.set_blocks(w.block_offsets())
    h.set_theta(w.theta0())
    cd = args.method == "cd"
    if cd:
        h.set_method(P.METHOD_CD)
        h.set_eps_mode(1)                     # Algorithm 1 keeps nu inside the root
    elif args.method != "ef":
        h.set_method(P.METHOD_NAIVE if args.method == "naive" else P.METHOD_NONE)
    step_bytes = w.algorithmic_bytes()
    if cd:                                    # + ghat r/w, gtilde r, gtilde r/w; Top-k: ghat_i is not rewritten
        step_bytes += 20 * w.d - (4 * w.n * w.d if w.compressor == W.TOPK else 0)
    elif args.method != "ef":                 # g is read, nothing is stored per worker
        step_bytes -= 8 * w.n * w.d
    if bf16:
        step_bytes -= 2 * w.n * w.d

    step_ptr = {"f32": h.step_ptr, "bf16": h.step_bf16_ptr, "f16": h.step_f16_ptr}[args.grad_dtype]

    def run(k0, count):
        for t in range(k0, k0 + count):
            step_ptr(dev_grads[t % nbuf].data_ptr(), stream)

    run(0, args.warmup)
    h.sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.warmup, args.steps)
    h.sync()                        # includes the update that the last step left to the next call
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    coords_per_s = w.n * w.d / (ms_per_step * 1e-3)

    # per-kernel durations: the same K steps again, every launch stamping a pair of HIP events with its begin and end
    h.profile(True)
    run(args.warmup + args.steps, args.steps)
    prof = h.profile_read()
    h.profile(False)
    kernels = {name: {"avg_us": ms * 1e3 / cnt, "launches_per_step": cnt / args.steps,
                      "us_per_step": ms * 1e3 / args.steps} for name, (ms, cnt) in prof.items()}
    # the dominant kernel among those that stream the step's arrays (the selection kernels between them work on
    # the candidate lists and carry no algorithmic bytes)
    streaming = [k for k in kernels if kernel_algorithmic_bytes(k, w.n, w.d, args.method) > 0] or list(kernels)
    dom = max(streaming, key=lambda k: kernels[k]["us_per_step"])
    dom_bytes = kernel_algorithmic_bytes(dom, w.n, w.d, args.method)
    if bf16 and dom in ("bs_pass", "bs_pass_update", "tk_pass1", "plain_update"):
        dom_bytes -= 2 * w.n * w.d
    dom_us = kernels[dom]["avg_us"]
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    traffic, traffic_source = measured_traffic(w.name, run_variant(args.method, args.grad_dtype, args.randk), dom)
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_source,
                "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_us": round(dom_us, 2)}
    if traffic:
        # bytes the counters saw per launch (in the separate counter run named above) over the duration measured
        # live here: the rate the memory system ran at
        roofline["traffic_gbs"] = round(traffic / (dom_us * 1e-6) / 1e9, 1)
        roofline["traffic_frac"] = round(roofline["traffic_gbs"] / HBM_PEAK_GBS, 4)
    step_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9

    # plain float4 copy on the same stream: what a trivial streaming kernel reaches on this chip, and
    # the launch that calibrates the HBM byte counters (it moves exactly 2 * probe bytes)
    copy_ceiling = None
    stream_ceiling = None
    if args.probe_mib > 0:
        count = args.probe_mib * (1 << 20) // 4
        src = torch.empty(count, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            P.probe_copy(dst, src)
        torch.cuda.synchronize()
        reps = 20
        c0 = time.perf_counter()
        for _ in range(reps):
            P.probe_copy(dst, src)
        torch.cuda.synchronize()
        copy_ceiling = {"gbs": round(2 * count * 4 * reps / (time.perf_counter() - c0) / 1e9, 1),
                        "bytes_per_launch": 2 * count * 4, "kernel": "probe_copy"}
        # the passes' own access pattern with nothing else (two arrays read, one of them written back in place):
        # the practical ceiling for the dominant kernel on this chip
        xs, gs = dst.view(8, count // 8), src.view(8, count // 8)
        for _ in range(3):
            P.probe_update(xs, gs)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(reps):
            P.probe_update(xs, gs)
        torch.cuda.synchronize()
        stream_ceiling = {"gbs": round(3 * count * 4 * reps / (time.perf_counter() - c0) / 1e9, 1),
                          "bytes_per_launch": 3 * count * 4, "kernel": "probe_update",
                          "pattern": "x[i][j] += g[i][j] in place, 8 rows"}
        del src, dst, xs, gs

    cpu = None
    if not args.no_cpu:
        from oracle import oracle as O
        ora = O.Oracle(w.d, w.n, compressor, kb, w.beta1, w.beta2, w.eps, w.lr,
                       method={"ef": O.EF, "cd": O.CD, "naive": O.NAIVE, "none": O.NONE}[args.method])
        if w.compressor == W.BLOCKSIGN and w.layer_blocks:
            ora.set_blocks(w.block_offsets())
        ora.set_theta(w.theta0())
        if cd:
            ora.set_eps_mode(1)
        ora.step(host_grads[0])                       # warm: first-touch of the oracle's arrays
        done, spent = 0, 0.0
        while done < 1 or spent < args.cpu_seconds:          # bounded by time, at least one step
            c0 = time.perf_counter()
            ora.step(host_grads[(done + 1) % nbuf])
            spent += time.perf_counter() - c0
            done += 1
        ora.close()
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = {"value": w.n * w.d / (spent / done), "unit": "coords/s", "cores": cores, "kind": "oracle",
               "sample": f"{done} full steps of {w.name} ({args.cpu_seconds:g} s budget) after one warm step, "
                         f"{spent / done * 1e3:.1f} ms/step"}

    out = {
        "metric": {"ef": "coords/sec (n*d) per COMP-AMS step", "cd": "coords/sec (n*d) per CD-Adam step",
                   "naive": "coords/sec (n*d) per naively compressed AMSGrad step",
                   "none": "coords/sec (n*d) per uncompressed AMSGrad step"}[args.method],
        "value": coords_per_s,
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "method": {"ef": "error_feedback", "cd": "cd_adam", "naive": "naive_compression",
                                                   "none": "no_compression"}[args.method], "gradients": args.grad_dtype, "n_workers": w.n, "d": w.d,
                   "compressor": "randk" if args.randk else "topk" if w.compressor == W.TOPK else "blocksign",
                   "k": w.k, "block": w.block, "layer_blocks": w.layer_blocks, "gradient_buffers": nbuf},
        "roofline": roofline,
        "step_algorithmic_gbs": round(step_gbs, 1),
        "step_frac_of_hbm_peak": round(step_gbs / HBM_PEAK_GBS, 4),
        "kernels": {k: {a: round(b, 3) for a, b in v.items()} for k, v in kernels.items()},
        "copy_ceiling": copy_ceiling,
        "stream_ceiling": stream_ceiling,
        "library_fingerprint": library_fingerprint(),
        "cpu_baseline": cpu,
    }
    h.destroy()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
