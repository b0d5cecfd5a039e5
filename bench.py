#!/usr/bin/env python3
"""Benchmark of the routing path on one MI355X.

One step = one pass of the whole path over one synthetic fleet, inputs already
in HBM: gr_build_status, gr_score_route over the incoming batch, gr_risk_scan
(status rebuilt from the refreshed lengths, flags, migration targets).

Prints ONE JSON line.  ``value`` is pair-estimates per second over the timed
steps: (incoming x instances) + (flagged x (instances - 1)) + one finish
estimate per held request in each of the two status builds, divided by wall
time.  ``roofline`` describes the kernel that took the most time, timed with
HIP events around each of its launches inside the timed region;
``cpu_baseline`` is the CPU reference timed on this machine's host cores on a
bounded sample of the same fleet.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
FP32_VECTOR_PEAK_TFLOPS = 157.3  # 256 CU x 128 lanes x 2 flop x 2.4 GHz (packed FMA)

# Algorithmic work per unit, independent of how the kernels are organised.
# Scoring, per (request, instance) pair: Eq. 2 from per-(instance, length) terms
# (one multiply-add = 2 flops) and the pair's part in the selections of Alg. 1
# (one comparison: the running least latency, which also decides feasibility
# because the feasible set is non-empty exactly when the least latency meets the
# deadline): 3 operations, counted as flops.
OPS_PER_PAIR = 3.0
# Status build, per held request: read prompt, generated, remaining (12 B), write
# finish (4 B) and one table entry (2 B sorted length + 8 B segment coefficients);
# the risk scan also reads the budget (4 B) and writes the flag (1 B).
BUILD_BYTES_PER_ENTRY = 26.0
SCAN_EXTRA_BYTES_PER_ENTRY = 5.0
# HBM bytes per launch of the dominant kernel come from the rocprofv3 counter passes summarised
# under profiles/ (not from this run): the summary of a workload carries a line
#   traffic-record: kernel=<name> fetch_bytes=<n> write_bytes=<n> sources_sha256=<hash>
# with the hash of the kernel sources the counters were taken with.  The figure is reported only
# while those sources are unchanged; otherwise null.
KERNEL_SOURCES = ("paper_2605_16867_amd/csrc/score.hip", "paper_2605_16867_amd/csrc/status.hip",
                  "paper_2605_16867_amd/csrc/common.h")


def sources_sha256() -> str:
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def recorded_traffic(workload: str, kernel: str):
    """(fetch + write bytes per launch, where it is from) or (None, why not)."""
    path = os.path.join(ROOT, "profiles", f"{workload}_step_all_kernels.md")
    if not os.path.exists(path):
        return None, "no counter summary for this workload under profiles/"
    for line in open(path):
        if line.startswith("traffic-record:"):
            kv = dict(item.split("=", 1) for item in line.split()[1:])
            if kv.get("kernel") != kernel:
                continue
            if kv.get("sources_sha256") != sources_sha256():
                return None, "kernel sources changed since the counters in profiles/ were taken"
            return int(kv["fetch_bytes"]) + int(kv["write_bytes"]), os.path.relpath(path, ROOT)
    return None, "no traffic record for this kernel under profiles/"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--blend", type=float, default=0.0,
                    help="weight of the black-box status (Sec. 3.3) after three rounds of synthetic observations")
    ap.add_argument("--batch-cap", action="store_true", help="per-instance caps on the decode batch (Sec. 3.1)")
    ap.add_argument("--feedback-chunk", type=int, default=0,
                    help="route the incoming batch with the status refreshed every so many requests")
    ap.add_argument("--latency-iters", type=int, default=100,
                    help="calls of gr_score_route timed one by one for the route-batch latency")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="heavy", help="tiny | mid | large | migrate | heavy")
    ap.add_argument("--prefixes", type=float, default=0.0,
                    help="mean number of cached prefixes per incoming request (Eq. 2's H); 0: none")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="target CPU time of the reference sample (0: skip)")
    return ap.parse_args()


def cpu_baseline(fl, pairs_route, pairs_migrate, entries, n_flagged, target_s):
    """Time the CPU reference (as it stands) on a bounded sample of this fleet and
    scale the two scanning legs to the whole step."""
    import oracle
    M = fl.n_inst
    rng = np.random.default_rng(0)
    t0 = time.perf_counter()
    sim = oracle.simulate(fl)
    t_sim = time.perf_counter() - t0
    R, na = len(fl.in_prompt), len(fl.act_prompt)
    budget = max(target_s - 2 * t_sim, 2.0) / 2

    def timed_route(n):
        idx = rng.choice(R, min(n, R), replace=False)
        t = time.perf_counter()
        sim.route(fl.in_prompt[idx], fl.in_len[idx], fl.in_budget[idx].astype(np.float64))
        return time.perf_counter() - t, len(idx)

    t_route = n_route = 0
    if R:
        t_probe, n_probe = timed_route(512)
        t_route, n_route = timed_route(int(max(512, n_probe * budget / max(t_probe, 1e-6))))
    t1 = time.perf_counter()
    sim2 = oracle.simulate(fl, fl.act_rem_refreshed)
    flag = np.flatnonzero(sim2.act_finish > fl.act_budget.astype(np.float64))
    t_sim2 = time.perf_counter() - t1
    t_mig = n_mig = 0
    if len(flag):
        def timed_mig(n):
            idx = rng.choice(flag, min(n, len(flag)), replace=False)
            inst_of = (np.searchsorted(fl.act_off, idx, side="right") - 1).astype(np.int32)
            c0 = fl.act_prompt[idx].astype(np.int64) + fl.act_gen[idx]
            t = time.perf_counter()
            sim2.route(c0, fl.act_rem_refreshed[idx], fl.act_budget[idx].astype(np.float64),
                       exclude=inst_of)
            return time.perf_counter() - t, len(idx)
        t_probe, n_probe = timed_mig(512)
        t_mig, n_mig = timed_mig(int(max(512, n_probe * budget / max(t_probe, 1e-6))))
    est = t_sim + t_sim2
    if n_route:
        est += t_route * R / n_route
    if n_mig:
        est += t_mig * len(flag) / n_mig
    total_pairs = pairs_route + len(flag) * (M - 1) + 2 * entries
    calls = {"gr_build_status": t_sim,
             "gr_score_route": (t_route * R / n_route) if n_route else 0.0,
             "gr_risk_scan": t_sim2 + ((t_mig * len(flag) / n_mig) if n_mig else 0.0)}
    return {
        "value": total_pairs / est, "unit": "pairs/s", "cores": oracle.threads(), "kind": "oracle",
        "seconds_per_call": calls,
        "sample": (f"both step-by-step simulations of all {M} instances ({t_sim + t_sim2:.2f} s), "
                   f"exhaustive scan of {n_route} of {R} incoming requests ({t_route:.2f} s) and of "
                   f"{n_mig} of {len(flag)} flagged requests ({t_mig:.2f} s), scan times scaled to the "
                   f"full batch; estimated CPU step {est:.1f} s"),
    }


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this path runs on one GPU; --gpus must be 1 "
              "(no collectives or sharding are part of this build)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_16867_amd import binding, workloads

    fl = workloads.make_fleet(workloads.spec(a.config))
    M, R = fl.n_inst, len(fl.in_prompt)
    na, nq = len(fl.act_prompt), len(fl.q_prompt)
    entries = na + nq
    dev = "cuda:0"
    torch.cuda.set_device(0)
    d = {k: torch.from_numpy(np.ascontiguousarray(getattr(fl, k))).to(dev) for k in
         ("act_off", "act_prompt", "act_gen", "act_rem", "act_rem_refreshed", "act_budget",
          "q_off", "q_prompt", "q_len", "in_prompt", "in_len", "in_budget")}
    h = binding.Fleet(fl.coef["delta"], fl.coef["alpha"], fl.coef["beta"], fl.coef["gamma"], fl.inst_class,
                      max(int(max(np.diff(fl.act_off) + np.diff(fl.q_off))), 1), int(fl.spec.max_len),
                      max(R, 1))

    fin = torch.empty(na, dtype=torch.float32, device=dev)
    inst = torch.empty(max(R, 1), dtype=torch.int32, device=dev)
    slack = torch.empty(max(R, 1), dtype=torch.float32, device=dev)
    flag = torch.empty(na, dtype=torch.uint8, device=dev)
    fin2 = torch.empty(na, dtype=torch.float32, device=dev)
    tgt = torch.empty(na, dtype=torch.int32, device=dev)
    tsl = torch.empty(na, dtype=torch.float32, device=dev)
    nfl = torch.zeros(1, dtype=torch.int32, device=dev)

    hits = None
    if a.prefixes > 0 and R:
        hits = [torch.from_numpy(x).to(dev) for x in workloads.cached_prefixes(fl, a.prefixes, seed=0)]

    variant = []
    if hits is not None:
        variant.append(f"prefixes({a.prefixes:g}/request)")
    if a.blend > 0:
        for w, ow, op, od in workloads.observed_status(fl, rounds=3, seed=0):
            h.gr_observe(w, *[torch.from_numpy(x).to(dev) for x in (ow, op, od)])
        h.gr_set_blend(a.blend)
        variant.append(f"blend({a.blend:g})")
    if a.batch_cap:
        h.gr_set_batch_cap(workloads.batch_caps(fl, seed=0))
        variant.append("batch-cap")
    if a.feedback_chunk > 0:
        variant.append(f"feedback(chunk={a.feedback_chunk})")

    def step():
        h.gr_build_status(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem"],
                          d["q_off"], d["q_prompt"], d["q_len"], fin)
        if R and a.feedback_chunk > 0:
            h.gr_route_feedback(a.feedback_chunk, d["in_prompt"], d["in_len"], d["in_budget"], inst, slack)
        elif R and hits is None:
            h.gr_score_route(d["in_prompt"], d["in_len"], d["in_budget"], inst, slack)
        elif R:
            h.gr_score_route_cached(d["in_prompt"], d["in_len"], d["in_budget"], hits[0], hits[1], hits[2],
                                    inst, slack)
        h.gr_risk_scan(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem_refreshed"],
                       d["q_off"], d["q_prompt"], d["q_len"], d["act_budget"],
                       flag, fin2, tgt, tsl, nfl)

    # launches of one step (the feedback variant repeats grouping, scoring and the status build per chunk)
    prof_slots = 32 + (16 * (-(-R // a.feedback_chunk)) if a.feedback_chunk > 0 else 0)
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    # before the timed region: the same steps with every kernel timed, for the breakdown and to
    # find the kernel the step spends most of its time in
    h.gr_profile_select(None)
    h.gr_profile_enable(prof_slots * a.steps)
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    launches_all = h.gr_profile_read_launches(prof_slots * a.steps)
    prof_all = {n: (sum(v), len(v)) for n, v in launches_all.items()}
    heaviest = max((n for n in prof_all if n.startswith(("k_tile", "k_build")) and prof_all[n][1]),
                   key=lambda n: prof_all[n][0])
    # timed region: HIP events around the launches of that kernel only (an event pair costs a few
    # microseconds of stream time: around each of the dozen launches of a step, about a tenth of it)
    h.gr_profile_select([heaviest])
    h.gr_profile_enable(prof_slots * a.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    launches = h.gr_profile_read_launches(prof_slots * a.steps)
    h.gr_profile_select(None)
    h.gr_profile_enable(0)
    for name, v in launches_all.items():
        if not launches.get(name):
            launches[name] = v
    prof = {n: (sum(v), len(v)) for n, v in launches.items()}

    # route-batch latency: gr_score_route alone on the warm handle, host clock around call + sync
    route_ms = []
    if R:
        h.gr_build_status(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem"],
                          d["q_off"], d["q_prompt"], d["q_len"], fin)
        for _ in range(a.latency_iters + 5):
            torch.cuda.synchronize()
            t = time.perf_counter()
            h.gr_score_route(d["in_prompt"], d["in_len"], d["in_budget"], inst, slack)
            torch.cuda.synchronize()
            route_ms.append((time.perf_counter() - t) * 1e3)
        route_ms = sorted(route_ms[5:])

    # a plain device-to-device copy of known size, outside the timed region: the
    # reference against which hardware memory counters of a profiled run are scaled
    cal_src = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    n_flagged = int(nfl.item())
    pairs_route, pairs_mig = R * M, n_flagged * (M - 1)
    pairs_step = pairs_route + pairs_mig + 2 * entries
    ms_step = dt / a.steps * 1e3

    kernels = {}
    for name, (ms, cnt) in prof.items():
        if not cnt:
            continue
        avg_ms = ms / cnt
        each = sorted(launches[name])
        k = {"avg_ms": avg_ms, "median_ms": each[len(each) // 2], "p99_ms": each[min(len(each) - 1, int(0.99 * len(each)))],
             "launches_per_step": cnt / a.steps}
        if name.startswith("k_tile"):
            pairs = (pairs_route if "route" in name else pairs_mig) / (cnt / a.steps)     # per launch
            k.update(bound="alu", pairs=pairs, pairs_per_s=pairs / (avg_ms * 1e-3),
                     achieved=pairs * OPS_PER_PAIR / (avg_ms * 1e-3) / 1e12,
                     peak=FP32_VECTOR_PEAK_TFLOPS, unit="TFLOP/s")
        elif name == "k_build" and cnt == 2 * a.steps:
            # two launches per step: plain build, and the scan's rebuild with budget + flag
            by = entries * (BUILD_BYTES_PER_ENTRY + SCAN_EXTRA_BYTES_PER_ENTRY / 2)
            k.update(bound="hbm", achieved=by / (avg_ms * 1e-3) / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
        if "achieved" in k:
            k["frac"] = k["achieved"] / k["peak"]
        kernels[name] = k
    dominant = max((n for n in kernels if "bound" in kernels[n]),
                   key=lambda n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"])
    dk = kernels[dominant]
    traffic, traffic_from = (recorded_traffic(a.config, dominant) if not variant
                             else (None, "variant run: no counters taken"))
    roofline = {"kernel": dominant, "bound": dk["bound"], "achieved": dk["achieved"], "peak": dk["peak"],
                "unit": dk["unit"], "frac": dk["frac"], "traffic": traffic, "traffic_from": traffic_from,
                "avg_launch_ms": dk["avg_ms"]}

    out = {
        "metric": "request x instance finish-estimates per second",
        "value": pairs_step / (dt / a.steps), "unit": "pairs/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "+".join([a.config] + variant),
                   "instances": M, "held_requests": entries,
                   "incoming": R, "flagged": n_flagged, "route_pairs": pairs_route,
                   "migration_pairs": pairs_mig},
        "roofline": roofline,
        "kernels": kernels,
    }
    if route_ms:
        out["route_batch_latency_ms"] = {
            "requests": R, "iters": len(route_ms), "median": route_ms[len(route_ms) // 2],
            "p99": route_ms[min(len(route_ms) - 1, int(0.99 * len(route_ms)))]}
    # achieved HBM rate as a share of the 8 TB/s peak: the streaming kernel on its algorithmic
    # bytes, the dominant kernel on the bytes the hardware counters saw
    out["hbm_pct_of_peak"] = {}
    if "frac" in kernels["k_build"]:
        out["hbm_pct_of_peak"]["k_build (algorithmic bytes)"] = 100.0 * kernels["k_build"]["frac"]
    if traffic is not None:
        out["hbm_pct_of_peak"][dominant + " (counter bytes from " + traffic_from + ")"] = (
            100.0 * traffic / (dk["avg_ms"] * 1e-3) / (HBM_PEAK_GBS * 1e9))
    if a.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(fl, pairs_route, pairs_mig, entries, n_flagged, a.cpu_seconds)
    h.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
