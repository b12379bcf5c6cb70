"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config {1..5}] [--no-cpu-baseline]

Default workload (--config 4, the one the metric is quoted on): allreduce, P=16384
virtual processes, f=4, 8 float64 values per process drawn N(0,1) (seed 4), 4096
failure scenarios (k uniform in 0..4 failed ranks, each failure before the operation
with probability 1/2, else during it at a uniform round).  One step = one pass of
the whole path over the batch, inputs resident in HBM: failure-scenario generation
(Philox), up-correction + tree phase + root's choice, retry attempts, broadcast
with correction into per-process receive buffers, and the validation kernels.
The other configurations (parity-test workloads, timed on request):
  1  reduce    P=8      f=1  4 x int64   288 scenarios (exhaustive sets x 32 payload seeds)
  2  allreduce P=64     f=2  8 x uint32  2081 scenarios (exhaustive sets), sum then bitwise or
  3  reduce    P=1024   f=3  16 x int64  65536 scenarios, a root per scenario
  5  allreduce P=2^20   f=8  1 x int64   1024 scenarios, a quarter of the failures during the operation
Prints ONE JSON line.
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

CONFIGS = {
    1: dict(kind="reduce", P=8, f=1, E=4, dtype="i64", ops=(0,), S=288, seed=1, bits=32, inop=0, roots=False,
            failures="exhaustive", repeat=32,
            text="reduce P=8 f=1 root 0 elems=4xi64 in [-2^31,2^31), exhaustive failure sets of size 0..1 x 32 payload "
                 "seeds (288 scenarios), all before the operation"),
    2: dict(kind="allreduce", P=64, f=2, E=8, dtype="u32", ops=(0, 1), S=2081, seed=2, bits=32, inop=0, roots=False,
            failures="exhaustive", repeat=1,
            text="allreduce P=64 f=2 elems=8xu32, exhaustive failure sets of size 0..2 (2081 scenarios), all before the "
                 "operation; a step runs the batch with the wrapping sum and again with the bitwise or"),
    3: dict(kind="reduce", P=1024, f=3, E=16, dtype="i64", ops=(0,), S=65536, seed=3, bits=41, inop=0, roots=True,
            failures="random",
            text="reduce P=1024 f=3 elems=16xi64 in [-2^40,2^40), a uniform root per scenario, k~U(0..3) failures "
                 "before the operation, S=65536 scenarios"),
    4: dict(kind="allreduce", P=16384, f=4, E=8, dtype="f64", ops=(0,), S=4096, seed=4, bits=0, inop=500, roots=False,
            failures="random",
            text="allreduce P=16384 f=4 elems=8xf64 N(0,1) S=4096 scenarios, k~U(0..4) failures, 1/2 pre-operational, "
                 "1/2 in-operation at a uniform round; per-process receive buffers materialised"),
    5: dict(kind="allreduce", P=1 << 20, f=8, E=1, dtype="i64", ops=(0,), S=1024, seed=5, bits=32, inop=250, roots=False,
            failures="random",
            text="allreduce P=2^20 f=8 elems=1xi64 in [-2^31,2^31) S=1024 scenarios (one batch: 8 GiB of inputs and 8 GiB "
                 "of receive buffers fit the HBM), k~U(0..8) failures, 1/4 in-operation at a uniform round"),
}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, choices=sorted(CONFIGS), help="workload (default 4, the headline one)")
    ap.add_argument("--scenarios", type=int, default=0, help="scenarios in the batch (default: the configuration's)")
    ap.add_argument("--lds-kib", type=int, default=0, help="ftred_plan flags (tuning knobs of the tree kernels; 0 = default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for HBM counters under rocprofv3)")
    ap.add_argument("--cpu-sample", type=int, default=0, help="scenarios timed on the CPU oracle (default: per configuration)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step into one HIP graph and time its replays (the launch-bound small "
                         "configurations; no per-kernel times, so no rooflines)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU (scenarios are independent; nothing is sharded); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2602_22445_amd import binding as ft
    from paper_2602_22445_amd import workloads as w

    ft.lib()                                   # fails loudly if the HIP library is missing or stale
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    c = CONFIGS[args.config]
    kind, P, f, E, seed = c["kind"], c["P"], c["f"], c["E"], c["seed"]
    is_all = kind == "allreduce"
    S = args.scenarios or c["S"]
    if c["failures"] == "exhaustive" and S != c["S"]:
        print("bench.py: configuration %d has a fixed batch (exhaustive failure sets)" % args.config, file=sys.stderr)
        sys.exit(2)
    dt = {"i64": ft.I64, "u32": ft.U32, "f64": ft.F64}[c["dtype"]]
    esz = ft.ELEM_SIZE[dt]
    plans = [ft.Plan(P, f, E, dt, op, args.lds_kib) for op in c["ops"]]
    plan = plans[0]
    rounds = plan.info.rounds_attempt if is_all else plan.info.rounds_reduce

    # ---- inputs (untimed), resident in HBM before the timed region
    t_in = time.time()
    if c["dtype"] == "f64":                    # generated on the host once and uploaded
        payload = torch.empty((S, P, E), dtype=torch.float64, device=dev)
        step_s = 256
        host = np.empty((step_s, P, E), dtype=np.float64)
        for s0 in range(0, S, step_s):
            n = min(step_s, S - s0)
            w.payload_normal(seed, n, P, E, scen0=s0, threads=16, out=host[:n])
            payload[s0:s0 + n].copy_(torch.from_numpy(host[:n]))
        del host
    else:                                      # the library's device generator (bit-identical to the host's)
        payload = ft.gen_payload_int(plan, seed, S, c["bits"])
    fail_rank = torch.empty((S, plan.F), dtype=torch.uint32, device=dev)
    fail_round = torch.empty((S, plan.F), dtype=torch.uint32, device=dev)
    root = None
    if c["failures"] == "exhaustive":          # fixed sets: resident, not generated per step
        fr9, fo9 = w.exhaustive_failure_sets(P, f)
        fail_rank.copy_(torch.from_numpy(np.repeat(fr9, c["repeat"], axis=0)))
        fail_round.copy_(torch.from_numpy(np.repeat(fo9, c["repeat"], axis=0)))
    torch.cuda.synchronize()
    t_in = time.time() - t_in

    ws = plan.workspace(S, dev)
    verdict = torch.empty(S, dtype=torch.uint32, device=dev)
    bufs = [None] * len(plans)
    red = [None] * len(plans)

    def step():
        nonlocal root
        if c["failures"] == "random":
            _, _, r = ft.gen_failures(plan, seed, S, inop_permille=c["inop"], rounds_per_attempt=rounds,
                                      protected=f + 1 if is_all else 0, want_root=c["roots"],
                                      fail_rank=fail_rank, fail_round=fail_round)
            root = r if c["roots"] else None
        for i, pl in enumerate(plans):
            if is_all:
                b = bufs[i] = ft.run_allreduce(pl, S, payload, fail_rank, fail_round, workspace=ws, buffers=bufs[i])
                ft.validate(pl, 1, S, payload, fail_rank, fail_round, b["result"], b["status"],
                            has_bitmap=b["has_bitmap"], per_process_out=b["per_process_out"], attempts=b["attempts"],
                            msgs=b["msgs"], workspace=ws, count=False, verdict=verdict)
            else:
                b = red[i] = ft.run_reduce(pl, S, payload, fail_rank, fail_round, root=root, workspace=ws, buffers=red[i])
                ft.validate(pl, 0, S, payload, fail_rank, fail_round, b["result"], b["status"], root=root,
                            msgs=b["msgs"], workspace=ws, count=False, verdict=verdict)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read, 1 GiB written
        src.zero_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del dst, src

    if args.graph:
        # the library only enqueues kernels on the caller's stream (workspace and outputs are the caller's, no
        # memset, no copy, no synchronisation), so the whole step records into one graph
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        last = bufs[-1] if is_all else red[-1]
        assert int((verdict.cpu().numpy() != 0).sum()) == 0, "validation rejected scenarios"
        attempts = last["attempts"].cpu().numpy().astype(np.int64) if is_all else np.ones(S, dtype=np.int64)
        process_rounds = int((attempts * rounds * P).sum()) * len(plans)
        print(json.dumps({
            "metric": "simulated process-rounds/sec and HBM GB/s (P=16384, f=4 allreduce), 1 GPU",
            "value": process_rounds * args.steps / (t1 - t0), "unit": "process-rounds/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": (t1 - t0) / args.steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": c["dtype"], "data": "synthetic",
            "config": {"workload": c["text"] + "; step = one replay of the captured HIP graph of "
                                   + ("generate failures + " if c["failures"] == "random" else "") + kind + " + validate",
                       "config_id": args.config, "scenarios": S, "plan_flags": args.lds_kib, "graph": True},
            "roofline": None, "cpu_baseline": None}))
        return

    # ---- timed region: exactly K steps, HIP events around every kernel launch
    ft.timing_begin(args.steps * 24 * len(plans))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    phases = ft.timing_end()

    # ---- what was computed
    last = bufs[-1] if is_all else red[-1]
    status = last["status"].cpu().numpy()
    n_invalid = int((verdict.cpu().numpy() != 0).sum())
    assert n_invalid == 0, "validation rejected %d scenarios" % n_invalid
    if is_all:
        attempts = last["attempts"].cpu().numpy().astype(np.int64)
        assert (status == 0).all()
    else:
        attempts = np.ones(S, dtype=np.int64)
    process_rounds = int((attempts * rounds * P).sum()) * len(plans)
    elapsed = t1 - t0
    value = process_rounds * args.steps / elapsed

    # ---- rooflines (algorithmic bytes per launch / average duration of the launch, HIP events)
    B = E * esz
    nrun = args.steps * len(plans)
    alg_bytes = {"tree_deep": S * P * B,                                   # every input read once
                 "val_partial": (2 if is_all else 1) * S * P * B}         # inputs (and receive buffers) read once
    if is_all:
        alg_bytes["bcast"] = S * P * B                                     # every receive buffer written once
    dom = max(alg_bytes, key=lambda k: phases[k][0])
    dom_ms = phases[dom][0] / max(phases[dom][1], 1)
    achieved = alg_bytes[dom] / (dom_ms * 1e-3) / 1e9
    kernels = {k: {"ms_avg": round(v[0] / max(v[1], 1), 4), "launches": v[1]} for k, v in phases.items() if v[1]}
    for k in alg_bytes:
        if k in kernels:
            kernels[k]["alg_GBs"] = round(alg_bytes[k] / (kernels[k]["ms_avg"] * 1e-3) / 1e9, 1)
    path_bytes = sum(alg_bytes.values()) * len(plans)
    # the operation itself, without generation and validation: all its kernels together
    op_ms = sum(phases[k][0] for k in ("check", "retry", "tree_deep", "tree_upper", "bcast")) / nrun
    op_bytes = (2 if is_all else 1) * S * P * B
    op_GBs = op_bytes / (op_ms * 1e-3) / 1e9
    # HBM bytes per launch from the counter runs kept under profiles/, while the kernels are still the
    # ones the counters were taken with
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic_allreduce_P16384_f4_S4096.txt")
    if args.config == 4 and os.path.exists(tfile) and S == 4096 and args.lds_kib == 0:
        from paper_2602_22445_amd import profile_summary
        per_kernel, sha = profile_summary.read_traffic(tfile)
        knames = {"tree_deep": ("fused_tree_kernel", "wave_tier_kernel"), "bcast": ("bcast_kernel",),
                  "val_partial": ("val_partial_kernel",)}[dom]
        if sha == profile_summary.source_hash():
            traffic = next((per_kernel[k] for k in knames if k in per_kernel), None)
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
        "dtype": c["dtype"],
        "data": "synthetic",
        "config": {"workload": c["text"] + "; step = " + ("generate failures + " if c["failures"] == "random" else "")
                               + kind + " + validate",
                   "config_id": args.config, "scenarios": S, "plan_flags": args.lds_kib},
        "process_rounds_per_step": process_rounds,
        "hbm_GBs_whole_step_algorithmic": path_bytes / (elapsed / args.steps) / 1e9,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic},
        # the reduce / allreduce proper: scenario check, retry attempts, tree tiers, broadcast (no generation, no validation)
        "operation_roofline": {"bound": "hbm", "what": kind + " kernels only (check, retry, tree tiers"
                                                       + (", broadcast)" if is_all else ")"),
                               "ms": op_ms, "algorithmic_bytes": op_bytes, "achieved": op_GBs, "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": op_GBs / HBM_PEAK_GBS,
                               "process_rounds_per_s": process_rounds / len(plans) / (op_ms * 1e-3)},
        "kernels": kernels,
        "input_setup_s": round(t_in, 2),
    }

    # ---- the CPU oracle on the host cores, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        import oracle
        odt = {"i64": oracle.I64, "u32": oracle.U32, "f64": oracle.F64}[c["dtype"]]
        op = c["ops"][-1]
        # a sample worth a few seconds on all cores, one sixteenth of it for the single-thread figure
        n = min(args.cpu_sample or {1: 288, 2: 2081, 3: 8192, 4: 4096, 5: 192}[args.config], S)
        n1 = max(1, n // 16)
        if c["dtype"] == "f64":
            x = payload[:n].cpu().numpy()      # generated on the host in the first place
        else:
            x = w.payload_int(seed, n, P, E, c["dtype"], c["bits"])
        fr = fail_rank[:n].cpu().numpy()
        fo = fail_round[:n].cpu().numpy()
        rt = root[:n].cpu().numpy() if root is not None else None

        def run(m, threads, full):
            if is_all:
                return oracle.allreduce_batch(P, f, x[:m], odt, op, m, fail_rank=fr[:m], fail_round=fo[:m],
                                              threads=threads, want_has=full, want_out=full)
            return oracle.reduce_batch(P, f, x[:m], odt, op, m, root=None if rt is None else rt[:m],
                                       fail_rank=fr[:m], fail_round=fo[:m], threads=threads)

        tc = time.perf_counter()
        o = run(n, 0, False)
        tc = time.perf_counter() - tc
        t1c = time.perf_counter()
        run(n1, 1, False)
        t1c = time.perf_counter() - t1c
        att_o = o["attempts"].astype(np.int64) if is_all else np.ones(n, dtype=np.int64)
        pr = int((att_o * rounds * P).sum())
        pr1 = int((att_o[:n1] * rounds * P).sum())
        # parity of the sample, untimed: every output of the operation
        m = min(n, 512 if P <= 16384 else 16)
        of = run(m, 0, True)
        res = last["result"][:m].cpu().numpy()
        assert np.array_equal(status[:m], of["status"]), "status differs from the oracle on the CPU sample"
        if c["dtype"] == "f64":
            tol = 1e-12 * np.abs(x[:m]).sum(axis=1)
            assert np.all(np.abs(res - of["result"]) <= tol), "result differs from the oracle on the CPU sample"
        else:
            assert np.array_equal(res, of["result"]), "result differs from the oracle on the CPU sample"
        assert np.array_equal(last["msgs"][:m].cpu().numpy(), of["msgs"]), "message counters differ from the oracle"
        if is_all:
            assert np.array_equal(attempts[:n], o["attempts"]), "attempts differ from the oracle"
            bits = np.unpackbits(last["has_bitmap"][:m].cpu().numpy().view(np.uint8), axis=1, bitorder="little")[:, :P]
            assert np.array_equal(bits, of["has"]), "holders differ from the oracle"
            assert np.array_equal(last["per_process_out"][:m].cpu().numpy(), of["out"]), "receive buffers differ from the oracle"
        out["cpu_baseline"] = {"value": pr / tc, "unit": "process-rounds/s", "cores": int(o["threads"]),
                               "kind": "oracle", "cpu_model": cpu_model(),
                               "value_1thread": pr1 / t1c,
                               "sample": "first %d of the %d scenarios on %d threads (%.1f s wall), first %d on one "
                                         "thread (%.1f s); the %s protocol only, WITHOUT validation and failure "
                                         "generation: compare with operation_roofline.process_rounds_per_s, not "
                                         "with value"
                                         % (n, S, int(o["threads"]), tc, n1, t1c, kind)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
