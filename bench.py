"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--scenarios S] [--no-cpu-baseline]

Workload: allreduce, P=16384 virtual processes, f=4, 8 float64 values per process
drawn N(0,1) (seed 4), 4096 failure scenarios (k uniform in 0..4 failed ranks, each
failure before the operation with probability 1/2, else during it at a uniform
round).  One step = one pass of the whole path over the batch, inputs resident in
HBM: failure-scenario generation (Philox), up-correction + tree phase + root's
choice, retry attempts, broadcast with correction into per-process receive
buffers, and the validation kernels.  Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--scenarios", type=int, default=4096)
    ap.add_argument("--lds-kib", type=int, default=0, help="ftred_plan flags (tuning knobs of the tree kernels; 0 = default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for HBM counters under rocprofv3)")
    ap.add_argument("--cpu-sample", type=int, default=2048, help="scenarios timed on the CPU oracle")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU (scenarios are independent; nothing is sharded); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2602_22445_amd import binding as ft
    from paper_2602_22445_amd import workloads as w

    ft.lib()                                   # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    P, f, E, S, seed = 16384, 4, 8, args.scenarios, 4
    plan = ft.Plan(P, f, E, ft.F64, ft.SUM, args.lds_kib)
    Ratt = plan.info.rounds_attempt

    # ---- inputs (untimed): payload generated on the host once, resident in HBM
    t_in = time.time()
    payload = torch.empty((S, P, E), dtype=torch.float64, device=dev)
    step_s = 256
    host = np.empty((step_s, P, E), dtype=np.float64)
    for s0 in range(0, S, step_s):
        n = min(step_s, S - s0)
        w.payload_normal(seed, n, P, E, scen0=s0, threads=16, out=host[:n])
        payload[s0:s0 + n].copy_(torch.from_numpy(host[:n]))
    torch.cuda.synchronize()
    t_in = time.time() - t_in

    ws = plan.workspace(S, dev)
    fail_rank = torch.empty((S, plan.F), dtype=torch.uint32, device=dev)
    fail_round = torch.empty((S, plan.F), dtype=torch.uint32, device=dev)
    verdict = torch.empty(S, dtype=torch.uint32, device=dev)
    bufs = None

    def step():
        nonlocal bufs
        ft.gen_failures(plan, seed, S, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1,
                        fail_rank=fail_rank, fail_round=fail_round)
        bufs = ft.run_allreduce(plan, S, payload, fail_rank, fail_round, workspace=ws, buffers=bufs)
        ft.validate(plan, 1, S, payload, fail_rank, fail_round, bufs["result"], bufs["status"],
                    has_bitmap=bufs["has_bitmap"], per_process_out=bufs["per_process_out"],
                    attempts=bufs["attempts"], msgs=bufs["msgs"], workspace=ws, count=False, verdict=verdict)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = payload[:1024].view(torch.float32)          # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del dst

    # ---- timed region: exactly K steps, HIP events around every kernel launch
    ft.timing_begin(args.steps * 16)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    phases = ft.timing_end()

    # ---- what was computed
    attempts = bufs["attempts"].cpu().numpy().astype(np.int64)
    status = bufs["status"].cpu().numpy()
    n_invalid = int((verdict.cpu().numpy() != 0).sum())
    assert n_invalid == 0, "validation rejected %d scenarios" % n_invalid
    assert (status == 0).all()
    process_rounds = int((attempts * Ratt * P).sum())
    elapsed = t1 - t0
    value = process_rounds * args.steps / elapsed

    # ---- roofline of the dominant kernel (algorithmic bytes per launch / average duration)
    B = E * 8
    alg_bytes = {
        "tree_deep": S * P * B,            # every input read once
        "bcast": S * P * B,                # every receive buffer written once
        "val_partial": 2 * S * P * B,      # inputs and receive buffers read once
    }
    dom = max(alg_bytes, key=lambda k: phases[k][0])
    dom_ms = phases[dom][0] / max(phases[dom][1], 1)
    achieved = alg_bytes[dom] / (dom_ms * 1e-3) / 1e9
    kernels = {k: {"ms_avg": round(v[0] / max(v[1], 1), 4), "launches": v[1]} for k, v in phases.items() if v[1]}
    for k in alg_bytes:
        kernels[k]["alg_GBs"] = round(alg_bytes[k] / (kernels[k]["ms_avg"] * 1e-3) / 1e9, 1)
    path_bytes = 4 * S * P * B             # the four passes above
    # HBM bytes per launch from the counter runs kept under profiles/, while the kernels are still the
    # ones the counters were taken with
    traffic = None
    tfile = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                         "hbm_traffic_allreduce_P16384_f4_S4096.txt")
    if os.path.exists(tfile) and S == 4096 and args.lds_kib == 0:
        from paper_2602_22445_amd import profile_summary
        per_kernel, sha = profile_summary.read_traffic(tfile)
        kname = {"tree_deep": "wave_tier_kernel", "bcast": "bcast_kernel", "val_partial": "val_partial_kernel"}[dom]
        if sha == profile_summary.source_hash() and kname in per_kernel:
            traffic = per_kernel[kname]
    out = {
        "metric": "simulated process-rounds/sec and HBM GB/s (P=16384, f=4 allreduce), 1 GPU",
        "value": value,
        "unit": "process-rounds/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "allreduce P=16384 f=4 elems=8xf64 N(0,1) S=%d scenarios, k~U(0..4) failures, "
                               "1/2 pre-operational, 1/2 in-operation at a uniform round; per-process receive "
                               "buffers materialised; step = generate failures + allreduce + validate" % S,
                   "scenarios": S, "plan_flags": args.lds_kib},
        "process_rounds_per_step": process_rounds,
        "hbm_GBs_whole_step_algorithmic": path_bytes / (elapsed / args.steps) / 1e9,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic},
        "kernels": kernels,
        "input_setup_s": round(t_in, 2),
    }

    # ---- the CPU oracle on the host cores, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        import oracle
        n = min(args.cpu_sample, S)
        x = payload[:n].cpu().numpy()
        fr = fail_rank[:n].cpu().numpy()
        fo = fail_round[:n].cpu().numpy()
        tc = time.perf_counter()
        o = oracle.allreduce_batch(P, f, x, oracle.F64, oracle.SUM, n, fail_rank=fr, fail_round=fo, threads=0,
                                   want_has=False, want_out=False)
        tc = time.perf_counter() - tc
        pr = int((o["attempts"].astype(np.int64) * Ratt * P).sum())
        res = bufs["result"][:n].cpu().numpy()
        tol = 1e-12 * np.abs(x).sum(axis=1)
        assert np.array_equal(o["attempts"], attempts[:n]) and np.all(np.abs(res - o["result"]) <= tol), \
            "GPU result differs from the oracle on the CPU sample"
        out["cpu_baseline"] = {"value": pr / tc, "unit": "process-rounds/s", "cores": int(o["threads"]),
                               "kind": "oracle",
                               "sample": "first %d of the %d scenarios, allreduce only (no validation), %.1f s wall"
                                         % (n, S, tc)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
