#!/usr/bin/env python3
"""Benchmark of the verify-and-recover block on one MI355X.

One step = one call of specsteer_verify_block (row log-sum-exp passes, ratio test, first
rejection, recovery distribution, sampling) over one batch of synthetic logits already
resident in HBM.  Prints ONE JSON line: verified draft positions per second on the headline
workload, the HBM roofline of the dominant kernel (row_lse) measured with HIP events on the
launch stream, the same figures for the one-pass schedule and for the other workloads, and
the float64 oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def describe(w) -> str:
    k = f"ragged K_b~U{{1..{w.k_max}}} k_max={w.k_max}" if w.ragged else f"K={w.k_max}"
    return (f"{w.name}: B={w.batch} {k} V={w.vocab} {w.dtype} sigma={w.sigma} T={w.temperature} "
            f"beta={w.beta} lambda={w.lam}")


def kernel_source_hash() -> str:
    """SHA-256 over the kernel sources the library is built from: a profile summary under profiles/
    records the hash of the build it measured, and only a summary of THIS build is quoted."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2603_16219_amd", "csrc")
    for name in sorted(os.listdir(src)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(src, name), "rb").read())
    h.update(open(os.path.join(ROOT, "include", "specsteer.h"), "rb").read())
    return h.hexdigest()[:16]


def read_traffic(workload: str):
    """HBM bytes per row_lse launch from the committed rocprofv3 --pmc summary of this workload, or None if
    there is none or it was taken on another build of the kernels."""
    path = os.path.join(ROOT, "profiles", f"verify_block_{workload}_pmc.txt")
    if not os.path.exists(path):
        return None, "no rocprofv3 --pmc summary for this workload"
    vals = {}
    for line in open(path):
        if ":" in line and line.split(":", 1)[0].strip() in ("kernel_source_sha256", "hbm_bytes_per_launch_read",
                                                             "hbm_bytes_per_launch_write"):
            k, v = line.split(":", 1)
            vals[k.strip()] = v.split()[0]
    if vals.get("kernel_source_sha256") != kernel_source_hash():
        return None, f"{os.path.basename(path)} was taken on another build of the kernels"
    if "hbm_bytes_per_launch_read" not in vals:
        return None, "summary holds no per-launch figure"
    return (float(vals["hbm_bytes_per_launch_read"]) + float(vals.get("hbm_bytes_per_launch_write", 0.0)),
            f"profiles/{os.path.basename(path)}")


def rows_view(torch, w, s, mode, dev):
    """Every row of a verify workload as a one-row sequence with no drafted position (views, no copy)."""
    n_rows = w.batch * (w.k_max + 1)
    r = {k: s[k].view(n_rows, 1, w.vocab) for k in ("G", "S_ctx", "S_noctx")}
    if mode == "draft_sample":
        r["G"] = r["S_noctx"] = r["S_ctx"]
    r["draft"] = torch.empty(n_rows, 0, dtype=torch.int32, device=dev)
    r["draft_len"] = None
    r["uniforms"] = s["uniforms"].reshape(n_rows, 1)
    return r


def measure_split(binding, w, sets, dev, *, steps, warmup) -> dict:
    """Deployment split: cloud top-k at one (seeded) row per sequence, then the edge resampling."""
    import torch

    B, V = w.batch, w.vocab
    esz = 2 if w.dtype == "bf16" else 4
    rows = [torch.randint(0, w.k_max + 1, (B,), generator=torch.Generator(dev).manual_seed(11 + i), device=dev,
                          dtype=torch.int32) for i in range(len(sets))]
    us = [s["uniforms"][:, -1].contiguous() for s in sets]

    def step(i):
        s = sets[i % len(sets)]
        idx, val = binding.cloud_topk(s["G"], s["S_noctx"], rows[i % len(sets)], beta=w.beta, topk=32)
        return binding.edge_resample(idx, val, s["S_ctx"], rows[i % len(sets)], us[i % len(sets)], beta=w.beta,
                                     temperature=w.temperature)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    # the cloud kernel alone: one pair of torch events on the current stream (the library launches there)
    # around a run of back-to-back launches, so that host-side call overhead hides behind the queue
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_timed = max(steps, 20)
    torch.cuda.synchronize()
    e0.record()
    for i in range(n_timed):
        s = sets[i % len(sets)]
        binding.cloud_topk(s["G"], s["S_noctx"], rows[i % len(sets)], beta=w.beta, topk=32)
    e1.record()
    e1.synchronize()
    kms = e0.elapsed_time(e1) / n_timed
    nbytes = 2.0 * B * V * esz
    return {"ms_per_step": ms, "rows_per_s": B / (ms * 1e-3), "kernel_ms": kms, "bytes": nbytes,
            "gbs": nbytes / (kms * 1e-3) / 1e9}


def bench_split(args, w, sets, dev) -> int:
    from paper_2603_16219_amd import binding

    m = measure_split(binding, w, sets, dev, steps=args.steps, warmup=args.warmup)
    out = {
        "metric": "top-32 downlink rows/sec", "value": m["rows_per_s"], "unit": "rows/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": m["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": describe(w), "mode": "cloud_topk", "topk": 32, "logits_dtype": w.dtype,
                   "kernel_source_sha256": kernel_source_hash()},
        "roofline": {"bound": "hbm", "kernel": "cloud_topk_kernel", "achieved": m["gbs"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": m["gbs"] / HBM_PEAK_GBS,
                     "traffic": None, "algorithmic_bytes_per_launch": m["bytes"], "avg_launch_ms": m["kernel_ms"]},
    }
    print(json.dumps(out), flush=True)
    return 0


def measure(binding, W, w, sets, dev, *, steps, warmup, mode="verify", full_rows=False, graph=False):
    """Time `steps` calls of the block on workload `w` (inputs already on the device) and the per-kernel stages
    of 20 further calls.  Returns the figures of one benchmark line; `state` holds what the parity check reuses."""
    import torch

    esz = 2 if w.dtype == "bf16" else 4
    B, kmax, V = w.batch, w.k_max, w.vocab
    rows_mode = mode in ("steer_rows", "draft_sample")
    if rows_mode:  # every row of the workload becomes a one-row sequence with no drafted position
        B, kmax = B * (kmax + 1), 0
    params = binding.make_params(B, kmax, V, W.torch_dtype(w.dtype), lam=w.lam,
                                 beta=0.0 if mode == "draft_sample" else w.beta, temperature=w.temperature,
                                 flags=(binding.SS_FLAG_GREEDY if mode == "greedy" else 0)
                                 | (binding.SS_FLAG_FULL_ROWS if full_rows else 0))
    t1 = binding.first_window(params)
    ws = torch.empty(max(256, binding.workspace_bytes(params)), dtype=torch.uint8, device=dev)
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    tok = torch.empty(B, dtype=torch.int32, device=dev)
    tlp = torch.empty(B, dtype=torch.float32, device=dev)

    def step(i, timed=False):
        s = sets[i % len(sets)]
        return binding.verify_block_raw(s["G"], s["S_ctx"], s["S_noctx"], s["draft"], s["draft_len"], s["uniforms"],
                                        params, acc, tok, tlp, None, None, ws, timed=timed)

    positions = [int(s["draft_len"].sum().item()) if s["draft_len"] is not None else B * max(kmax, 1) for s in sets]
    run = step
    if graph:
        # the step's launches (kernels only: the library enqueues no memset, copy or allocation) captured once
        # per input set and replayed: what a launch-bound caller (small batches) would do
        step(0)
        torch.cuda.synchronize()
        graphs = []
        for j in range(len(sets)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(j)
            graphs.append(g)

        def run(i):
            graphs[i % len(sets)].replay()

    for i in range(warmup):
        run(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        run(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    pos_total = sum(positions[i % len(sets)] for i in range(steps))
    ms_per_step = elapsed / steps * 1e3

    # per-kernel durations: HIP events recorded on the launch stream, inside the library
    n_timed = min(steps, 20)
    stage = {k: 0.0 for k in binding.STAGES}
    lse_bytes = step_bytes = bonus_frac = rows_scored = 0.0
    for i in range(n_timed):
        ms = step(i, timed=True)
        for k in stage:
            stage[k] += ms[k] / n_timed
        s = sets[i % len(sets)]
        K = s["draft_len"] if s["draft_len"] is not None else torch.full((B,), kmax, dtype=torch.int32, device=dev)
        n_bonus = int((acc == K).sum().item())
        # rows the schedule scores: the first window for everyone, the rest for sequences not rejected inside it
        in_play = (K > t1) & (acc >= t1)
        rows = int(torch.clamp(K, max=t1).sum().item()) + int((K - t1)[in_play].sum().item())
        rows_scored += rows / n_timed
        # row pass: two rows of V logits per scored position
        lse_bytes += 2.0 * rows * V * esz / n_timed
        # whole step, unique bytes: the row passes, the S_ctx recovery row of every sequence, and the
        # G / S_noctx bonus rows of fully accepted sequences (a rejected row was already read by a row pass)
        step_bytes += (2.0 * rows + B + 2.0 * n_bonus) * V * esz / n_timed
        bonus_frac += n_bonus / B / n_timed
    n_lse = 2 if (not rows_mode and t1 < kmax) else 1  # launches of the row-pass kernel per step
    # a stage that launches nothing still measures the ~5 us of its event pair: only passes that ran are counted
    lse_ms = stage["row_pass1"] + (stage["row_pass2"] if n_lse == 2 else 0.0)
    lse_gbs = lse_bytes / (lse_ms * 1e-3) / 1e9 if lse_ms > 0 else 0.0
    if rows_mode:
        # no row pass: the recovery sweep is the dominant (only) kernel; it reads 3 rows per row, 1 when beta = 0
        per_row = (1 if mode == "draft_sample" else 3) * V * esz
        lse_bytes = step_bytes = float(B) * per_row
        lse_gbs = lse_bytes / (stage["recover"] * 1e-3) / 1e9
    return {
        "value": pos_total / elapsed, "ms_per_step": ms_per_step, "positions": positions, "first_window": t1,
        "rows_scored": rows_scored, "bonus_frac": bonus_frac, "stage": stage, "n_lse": n_lse,
        "lse_bytes_per_launch": lse_bytes / n_lse, "lse_gbs": lse_gbs,
        "avg_launch_ms": stage["recover"] if rows_mode else lse_ms / n_lse,
        "step_bytes": step_bytes, "step_gbs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "state": (params, ws, acc, tok, tlp), "batch": B, "k_max": kmax,
    }


def brief(m) -> dict:
    """The figures of `measure` that a sub-record of the JSON line carries."""
    return {"us_per_step": round(m["ms_per_step"] * 1e3, 2), "positions_per_s": round(m["value"], 1),
            "first_window": m["first_window"], "rows_scored_per_step": round(m["rows_scored"], 1),
            "row_pass_GB/s": round(m["lse_gbs"], 1), "row_pass_frac_of_peak": round(m["lse_gbs"] / HBM_PEAK_GBS, 4),
            "row_pass_launches": m["n_lse"],
            "whole_step_GB/s": round(m["step_gbs"], 1), "whole_step_frac_of_peak": round(m["step_gbs"] / HBM_PEAK_GBS, 4),
            "stages_us": {k: round(v * 1e3, 2) for k, v in m["stage"].items()}}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c4", help="c1..c5 (c4 is the configuration the target is quoted on)")
    ap.add_argument("--sets", type=int, default=2, help="rotating input sets")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the one-pass schedule, the other modes and the other workloads (the short sub-records of the line)")
    ap.add_argument("--dtype", choices=["bf16", "f32"], default=None,
                    help="store the workload's logits in this type instead of its own (same recipe, rounded to it)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a HIP graph of the step instead of direct launches (verify modes only)")
    ap.add_argument("--lam", type=float, default=None, help="override the verification threshold")
    ap.add_argument("--mode", default="verify", choices=["verify", "greedy", "steer_rows", "draft_sample", "cloud_topk"],
                    help="verify: the block (default, the headline metric); greedy: same with argmax recovery; "
                         "steer_rows: always-on steering, Eq. 8 + one draw on every row of the workload; "
                         "draft_sample: softmax sampling of every S_ctx row (the drafting step); "
                         "cloud_topk: the deployment split, top-32 of h_LLM - beta*h_SLM^- at one row per sequence "
                         "followed by the edge-side resampling")
    ap.add_argument("--full-rows", action="store_true",
                    help="one-pass schedule: score every valid row even after a sequence's first rejection")
    ap.add_argument("--dense", action="store_true", help="ignore the length array of a ragged workload (K_b = k_max)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the block shards by sequence with no "
              "communication; multi-GPU figures are not part of it). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch

    from paper_2603_16219_amd import binding, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    binding.library()
    dev = torch.device("cuda:0")
    w = W.WORKLOADS[args.workload]
    if args.lam is not None:
        import dataclasses
        w = dataclasses.replace(w, lam=args.lam)
    if args.dtype is not None and args.dtype != w.dtype:
        import dataclasses
        w = dataclasses.replace(w, dtype=args.dtype, name=f"{w.name}@{args.dtype}")

    def make_sets(wl, n):
        sets_ = [W.generate(wl, dev, seed_shift=i) for i in range(max(1, n))]
        if args.dense:
            for s_ in sets_:
                s_["draft_len"] = None
        return sets_

    sets = make_sets(w, args.sets)
    V = w.vocab
    if args.mode == "cloud_topk":
        return bench_split(args, w, sets, dev)
    rows_mode = args.mode in ("steer_rows", "draft_sample")
    if rows_mode:
        sets = [rows_view(torch, w, s_, args.mode, dev) for s_ in sets]

    if args.calibrate_copy:
        # a plain elementwise copy of known size: reads 1 GiB, writes 1 GiB per launch
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    m = measure(binding, W, w, sets, dev, steps=args.steps, warmup=args.warmup, mode=args.mode,
                full_rows=args.full_rows, graph=args.graph)
    B, kmax = m["batch"], m["k_max"]
    traffic, traffic_note = (read_traffic(w.name) if args.mode == "verify" and not args.full_rows and not args.graph
                             and args.lam is None and not args.dense else (None, "only quoted for the default call"))
    out = {
        "metric": "verified draft positions/sec" if not rows_mode else "sampled rows/sec",
        "value": m["value"],
        "unit": "positions/s" if not rows_mode else "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": describe(w), "mode": args.mode, "logits_dtype": w.dtype, "input_sets": len(sets),
                   "positions_per_step": m["positions"][0],
                   "rows_per_step": m["positions"][0] + B if not rows_mode else B,
                   "bonus_fraction": round(m["bonus_frac"], 4),
                   "first_window": m["first_window"], "rows_scored_per_step": round(m["rows_scored"], 1),
                   "launch": "hip graph replay" if args.graph else "direct",
                   "kernel_source_sha256": kernel_source_hash()},
        "roofline": {
            "bound": "hbm", "kernel": "accept_recover_kernel" if rows_mode else "row_lse_kernel",
            "achieved": m["lse_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": m["lse_gbs"] / HBM_PEAK_GBS,
            "traffic": traffic, "traffic_source": traffic_note,
            "algorithmic_bytes_per_launch": m["lse_bytes_per_launch"], "avg_launch_ms": m["avg_launch_ms"],
            "launches_per_step": m["n_lse"],
        },
        "stages_ms": {k: round(v, 5) for k, v in m["stage"].items()},
        "whole_step": {"algorithmic_bytes": m["step_bytes"], "GB/s": m["step_gbs"],
                       "frac_of_peak": m["step_gbs"] / HBM_PEAK_GBS},
    }

    params, ws, acc, tok, tlp = m["state"]
    if not args.no_cpu_baseline and rows_mode:
        print("bench.py: --mode steer_rows / draft_sample report no cpu_baseline (use --no-cpu-baseline to silence)",
              file=sys.stderr)
    if not args.no_cpu_baseline and not rows_mode:
        import oracle
        import parity

        oracle.build()
        s = sets[0]
        # bounded sample: whole sequences, at most ~6e8 exponentials per pass (the whole batch for c1-c4)
        exps_per_seq = (2.0 * m["positions"][0] / B + 1.5) * V
        nseq = int(max(1, min(B, 6e8 // max(exps_per_seq, 1))))
        # every host core this process may use: the machine's count, capped by the share the environment grants
        # (OMP_NUM_THREADS, CPU affinity); both counts are stated
        host_cpus = os.cpu_count() or 1
        share = min(host_cpus, len(os.sched_getaffinity(0)), oracle.max_threads())
        threads = max(1, min(share, nseq))
        seqs = torch.arange(nseq, device=dev)
        host = {k: (None if v is None else v[:nseq].cpu()) for k, v in s.items()}
        # the oracle stops at the first rejection as Algorithm 1 does, so one pass is short: repeat it
        # (same inputs) until about a second of wall time has gone by and report the median pass
        walls = []
        while len(walls) < 9 and (sum(walls) < 1.0 or len(walls) < 3):
            t0 = time.perf_counter()
            ora = oracle.verify_block(host["G"], host["S_ctx"], host["S_noctx"], host["draft"], host["uniforms"],
                                      lam=w.lam, beta=w.beta, temperature=w.temperature, draft_len=host["draft_len"],
                                      want_recovery_logprobs=False, num_threads=threads, greedy=args.mode == "greedy")
            walls.append(time.perf_counter() - t0)
        cpu_s = sorted(walls)[len(walls) // 2]
        t0 = time.perf_counter()  # and one pass on a single thread
        oracle.verify_block(host["G"], host["S_ctx"], host["S_noctx"], host["draft"], host["uniforms"],
                            lam=w.lam, beta=w.beta, temperature=w.temperature, draft_len=host["draft_len"],
                            want_recovery_logprobs=False, num_threads=1, greedy=args.mode == "greedy")
        cpu_1 = time.perf_counter() - t0
        cpu_pos = int(host["draft_len"].sum().item()) if host["draft_len"] is not None else nseq * kmax
        out["cpu_baseline"] = {
            "value": cpu_pos / cpu_s, "unit": "positions/s", "cores": threads, "kind": "oracle",
            "value_one_thread": cpu_pos / cpu_1, "host_cpu_count": host_cpus, "cpu_share_of_this_process": share,
            "sample": f"first {nseq} of {B} sequences of {w.name} ({cpu_pos} positions), float64 oracle, "
                      f"{threads} OpenMP threads over sequences (the box shows {host_cpus} CPUs, this process may use "
                      f"{share}), median of {len(walls)} passes of {cpu_s:.3f} s wall "
                      f"({sum(walls) * threads:.0f} CPU-seconds in all)",
        }
        # parity of the same step against the oracle, reported beside the timing: the step as timed, plus a
        # second call that also asks for the per-position log-probs (which takes the one-pass schedule)
        parity.attach_recheck(ora, oracle, host["G"], host["S_ctx"], host["S_noctx"], host["draft"], host["draft_len"],
                              lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=args.mode == "greedy")
        binding.verify_block_raw(s["G"], s["S_ctx"], s["S_noctx"], s["draft"], s["draft_len"], s["uniforms"], params,
                                 acc, tok, tlp, None, None, ws)
        dlp = torch.empty(B, kmax, 2, dtype=torch.float32, device=dev)
        acc2, tok2, tlp2 = torch.empty_like(acc), torch.empty_like(tok), torch.empty_like(tlp)
        binding.verify_block_raw(s["G"], s["S_ctx"], s["S_noctx"], s["draft"], s["draft_len"], s["uniforms"], params,
                                 acc2, tok2, tlp2, None, dlp, ws)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc2) and torch.equal(tok, tok2), "the two schedules disagree"
        rep = parity.compare({"accepted_len": acc, "next_token": tok, "next_token_logprob": tlp,
                              "draft_logprobs": dlp}, ora, s["uniforms"], s["draft_len"], seqs=seqs)
        out["parity"] = rep
        del host, ora, dlp

    extras = (args.mode == "verify" and not args.no_extras and not args.graph and not args.full_rows
              and args.lam is None and args.dtype is None and not args.dense)
    if extras:
        # the same workload on the one-pass schedule (every valid row scored), a short second loop
        fr = measure(binding, W, w, sets, dev, steps=min(args.steps, 20), warmup=min(args.warmup, 5), full_rows=True)
        out["full_rows"] = brief(fr)
        # the modes that run on the same kernels, on the same logits: short loops
        short = dict(steps=min(args.steps, 20), warmup=min(args.warmup, 5))
        modes = {}
        gm = measure(binding, W, w, sets, dev, mode="greedy", **short)
        modes["greedy"] = {"us_per_step": round(gm["ms_per_step"] * 1e3, 2), "positions_per_s": round(gm["value"], 1)}
        for md in ("steer_rows", "draft_sample"):
            rm = measure(binding, W, w, [rows_view(torch, w, s_, md, dev) for s_ in sets], dev, mode=md, **short)
            modes[md] = {"us_per_step": round(rm["ms_per_step"] * 1e3, 2), "rows_per_s": round(rm["value"], 1),
                         "kernel_us": round(rm["avg_launch_ms"] * 1e3, 2), "kernel_GB/s": round(rm["lse_gbs"], 1),
                         "kernel_frac_of_peak": round(rm["lse_gbs"] / HBM_PEAK_GBS, 4)}
            del rm
        sm = measure_split(binding, w, sets, dev, **short)
        modes["cloud_topk"] = {"us_per_step": round(sm["ms_per_step"] * 1e3, 2), "rows_per_s": round(sm["rows_per_s"], 1),
                               "kernel_us": round(sm["kernel_ms"] * 1e3, 2), "kernel_GB/s": round(sm["gbs"], 1),
                               "kernel_frac_of_peak": round(sm["gbs"] / HBM_PEAK_GBS, 4)}
        out["modes"] = modes
        del fr, m, gm
        del sets, ws, acc, tok, tlp
        torch.cuda.empty_cache()
        # the other workloads: microseconds per step in the launch configuration the tests verify
        out["configs"] = {}
        for name in ("c1", "c2", "c3", "c4", "c5"):
            if name == w.name:
                continue
            wl = W.WORKLOADS[name]
            osets = make_sets(wl, 2)
            om = measure(binding, W, wl, osets, dev, steps=min(args.steps, 30), warmup=min(args.warmup, 5))
            rec = brief(om)
            rec["workload"] = describe(wl)
            if wl.batch * wl.k_max * 2 * wl.vocab * (2 if wl.dtype == "bf16" else 4) < (96 << 20):
                rec["note"] = "launch/latency-bound (under 100 MB per call): quoted as latency, fractions are not meaningful"
            out["configs"][name] = rec
            del osets, om
            torch.cuda.empty_cache()

    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
