#!/usr/bin/env python3
"""Throughput of the exponential-race verification hot path on one MI355X.

One "step" is one pass of the whole hot path (race kernel + finishing kernel) over one batch of synthetic logits
that are already resident in HBM.  The headline line is measured on the largest of the benchmark workloads
(B=256, k=16, V=152064, fp32: 5.14 GB of logits per step); the same run then measures the three other full-size
workloads (1: sequence bf16, 3: multi-draft bf16, 4: tree bf16) and reports them under "per_workload", each
with its own step time, race-kernel time, HBM fraction, plain-read figure and oracle check.  Prints ONE JSON line.

Timing.  `value` comes from a wall-clock loop over whole steps (the verify entry point), bracketed by device
synchronisation.  The race kernel's own duration is measured afterwards, in the same process and on the same
stream, with HIP events around a batch of back-to-back launches of the race stage (ersd_race_stage_races, the first
of the two stage entry points that together are exactly ersd_race_verify*), at least 20 of them whatever --steps is;
a second loop brackets single launches for the minimum and the median.  Input buffers rotate over several distinct
sets so that the 256 MB on-die cache cannot serve the reads.
"""
import argparse
import json
import sys
import time

import torch

PEAK_HBM_GBS = 8000.0
ARITHMETIC = "u32+f32 filter, f64 decide"  # u32 Philox + f32 bound filter on every token, f64 scores where f32 cannot decide

# HBM bytes per race-kernel launch from rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE, each scaled by what the same
# counter reads for a 1 GiB copy); NOT measured in this run: the figures of the summaries under profiles/, which
# name the commands that produced them.
PROFILED_TRAFFIC_BYTES = {1: 279967334, 2: 5141426511, 3: 1117813011, 4: 1049643334}
PROFILE_FILE = {1: "profiles/race_kernel_seq_B64_k8_V128256_bf16.md", 2: "profiles/race_kernel_seq_B256_k16_V152064_f32.md",
                3: "profiles/race_kernel_multi_B32_m8_k8_V128256_bf16.md", 4: "profiles/race_kernel_tree_B16_N64_V256000_bf16.md"}


def make_sets(w, dev, count):
    """`count` distinct input sets of one workload: set 0 is the workload's own recipe, the others add 1 % noise
    (a permutation of rows would alias in the cache)."""
    from paper_2504_15475_amd import workloads as wl
    base = wl.make_inputs(w, dev)
    sets = [base]
    for i in range(1, max(1, count)):
        g = torch.Generator(device=dev).manual_seed(5000 + i)
        noise = lambda x: (x.float() + 0.01 * torch.randn(x.shape, generator=g, device=dev)).to(x.dtype).contiguous()
        s = dict(draft=noise(base["draft"]), target=noise(base["target"]))
        if "parent" in base:
            s["parent"] = base["parent"]
        sets.append(s)
    return sets


def measure_verify(w, sets, args, dev, timed_baseline):
    """One full-size workload through the verify path -> dict(value, ms_per_step, roofline, check[, cpu_baseline])."""
    from paper_2504_15475_amd import race, workloads as wl
    variant = {"sequence": race.VARIANT_SEQUENCE, "multi": race.VARIANT_MULTI, "tree": race.VARIANT_TREE}[w.variant]
    calls = [race.PreparedVerify(variant, s["draft"], s["target"], w.temperature, w.seed, s.get("parent")) for s in sets]
    torch.cuda.synchronize()
    nset = len(calls)

    for i in range(args.warmup):
        calls[i % nset].run()
    torch.cuda.synchronize()

    # 1. whole steps, wall clock: the headline throughput
    K = args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        calls[i % nset].run()
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    ms_per_step = total_s * 1e3 / K

    # 2. the race kernel alone: HIP events around a batch of back-to-back launches, then around single launches
    n_ev = max(20, args.event_launches)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def batch(n):
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            calls[i % nset].run_races()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    rough = batch(n_ev)
    n_ev = max(n_ev, min(400, int(20.0 / rough)))  # about 20 ms of launches, so that a short kernel is not timed on 2 ms
    batch(n_ev)  # this measurement's own warm-up: the wall-clock loop above may have been short, and the device idles
    kernel_ms = batch(n_ev)  # (and clocks down) whenever the host is busy with the oracle
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(n_ev, 64))]
    for i, (a0, a1) in enumerate(pairs):
        a0.record()
        calls[i % nset].run_races()
        a1.record()
        calls[i % nset].run_accept()
    torch.cuda.synchronize()
    single = sorted(a0.elapsed_time(a1) for a0, a1 in pairs)

    # 3. context: the same tensors read once by a kernel that does nothing else, with the race kernel's loads and
    # launch shape, timed the same way
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    for i in range(8):
        race.read_probe(sets[i % nset]["draft"], sets[i % nset]["target"], sink)
    torch.cuda.synchronize()
    e0.record()
    for i in range(n_ev):
        race.read_probe(sets[i % nset]["draft"], sets[i % nset]["target"], sink)
    e1.record()
    torch.cuda.synchronize()
    probe_ms = e0.elapsed_time(e1) / n_ev

    algo_bytes = w.logit_bytes
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    out = {
        "workload": w.name, "description": wl.describe(w), "race_elements_per_step": w.race_elements,
        "logit_dtype": "bf16" if w.elem_bytes == 2 else "fp32",
        "value": w.race_elements * K / total_s, "unit": "elements/s", "steps": K, "ms_per_step": ms_per_step,
        "roofline": {
            "bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": PROFILED_TRAFFIC_BYTES.get(w.index),
            "traffic_source": (PROFILE_FILE[w.index] + " (rocprofv3 --pmc, not measured in this run)")
            if w.index in PROFILE_FILE else None,
            "kernel": "race_kernel", "timing": f"HIP events around {n_ev} back-to-back launches of the race stage",
            "launches_timed": n_ev, "kernel_ms_avg": round(kernel_ms, 5),
            "single_launch_ms": {"avg": round(sum(single) / len(single), 5), "min": round(single[0], 5),
                                 "median": round(single[len(single) // 2], 5),
                                 "note": "one launch between two events; includes the events' own few microseconds"},
            "algorithmic_bytes_per_launch": algo_bytes,
            "whole_step_frac": round(algo_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "plain_read_same_shape": {"ms": round(probe_ms, 5), "GB/s": round(algo_bytes / (probe_ms * 1e-3) / 1e9, 1),
                                      "race_kernel_vs_plain_read": round(probe_ms / kernel_ms, 4)},
        },
    }
    out["_oracle"] = lambda: oracle_side(w, sets[0], calls[0], variant, timed_baseline)
    return out


def add_oracle_side(rec):
    """The host-side part of one workload's record, run after every GPU measurement of the run is done."""
    base_out, check = rec.pop("_oracle")()
    rec["check"] = check
    if base_out is not None:
        rec["cpu_baseline"] = base_out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=2,
                    help="index into the five benchmark workloads for the headline line (default 2, the largest); "
                         "5 = the tree of workload 4 verified as Algorithm 5 states it (children of a context = "
                         "first arrivals of one race)")
    ap.add_argument("--also", type=str, default=None,
                    help="comma-separated workloads measured after the headline one and reported under per_workload "
                         "(default: 1,3,4 with the default headline workload, none otherwise; '' for none)")
    ap.add_argument("--buffers", type=int, default=4, help="distinct input sets rotated through (cache defeat)")
    ap.add_argument("--event-launches", type=int, default=48,
                    help="launches of the race kernel timed with HIP events (at least 20 are always timed)")
    ap.add_argument("--entry", choices=["verify", "sample", "gsd", "calibrate"], default="verify",
                    help="verify: the fused draft+target races (default, the headline metric); sample: the one-model "
                         "entry point on the workload's target logits (how a serving loop calls the race); gsd: the "
                         "comparison method (ersd_gsd_verify) on the same logits, sequence workloads only; calibrate: "
                         "a plain 1 GiB device-to-device copy, to be run under rocprofv3 --pmc so that the HBM byte "
                         "counters can be scaled by a kernel of known traffic")
    ap.add_argument("--npos", type=int, default=0,
                    help="with --entry sample: positions per call (0 = all target rows at once; 1 = the drafting call)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus must be 1",
              file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        return 2

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.entry == "calibrate":
        return calibrate(dev)
    from paper_2504_15475_amd import race, workloads as wl
    race.lib()
    if args.workload == 5:
        if args.entry == "gsd":
            return bench_gsd_tree(args, wl.ARRIVAL_TREE, dev)
        return bench_arrival_tree(args, wl.ARRIVAL_TREE, dev)
    w = wl.WORKLOADS[args.workload]
    if args.entry == "sample":
        return bench_sample(args, w, dev)
    if args.entry == "gsd":
        return bench_gsd(args, w, dev)

    also = args.also if args.also is not None else ("1,3,4" if args.workload == 2 else "")
    others = [int(x) for x in also.split(",") if x.strip() != ""]

    # The inputs of every workload of the run are generated first and stay allocated to the end (30 GB for the default
    # run): memory that a process has freed and allocates again is read measurably slower on this machine (a plain
    # read of 1.1 GB takes 172 us instead of 165), which would favour whichever workload came first.
    inputs = {args.workload: make_sets(w, dev, args.buffers)}
    failed = []  # a secondary workload that cannot be measured is reported as such; the headline line still stands
    for i in others:
        try:
            inputs[i] = make_sets(wl.WORKLOADS[i], dev, args.buffers)
        except Exception as e:  # noqa: BLE001
            failed.append({"workload": wl.WORKLOADS[i].name, "error": f"{type(e).__name__}: {e}"})
    torch.cuda.synchronize()
    head = measure_verify(w, inputs[args.workload], args, dev, timed_baseline=not args.no_cpu_baseline)
    per = []
    for i in others:
        if i not in inputs:
            continue
        try:
            per.append(measure_verify(wl.WORKLOADS[i], inputs[i], args, dev, timed_baseline=False))
        except Exception as e:  # noqa: BLE001
            failed.append({"workload": wl.WORKLOADS[i].name, "error": f"{type(e).__name__}: {e}"})
    add_oracle_side(head)
    for rec in list(per):
        try:
            add_oracle_side(rec)
        except Exception as e:  # noqa: BLE001
            rec.pop("_oracle", None)
            rec["check"] = {"error": f"{type(e).__name__}: {e}"}

    out = {
        "metric": "race_elements_per_sec", "value": head["value"], "unit": "elements/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": ARITHMETIC, "data": "synthetic",
        "config": {"workload": head["workload"], "description": head["description"],
                   "race_elements_per_step": head["race_elements_per_step"], "logit_dtype": head["logit_dtype"],
                   "input_buffer_sets": args.buffers, "philox_rounds": race.philox_rounds(),
                   "issue": "verify entry point (value); race stage entry point (roofline)"},
        "roofline": head["roofline"],
        "check": head["check"],
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    if per:
        out["per_workload"] = [
            {k: x[k] for k in ("workload", "description", "logit_dtype", "race_elements_per_step", "value", "unit",
                               "ms_per_step", "roofline", "check")} for x in per]
        fracs = {x["workload"]: x["roofline"]["frac"] for x in [head] + per}
        out["min_frac"] = {"workload": min(fracs, key=fracs.get), "frac": min(fracs.values()),
                           "over": "race kernel, the headline workload and per_workload"}
    if failed:
        out["per_workload_failed"] = failed
    print(json.dumps(out), flush=True)
    return 0


def calibrate(dev, mib=1024, reps=3):
    """A device-to-device copy of known size: each copy reads `mib` MiB and writes `mib` MiB, so the ratio of a byte
    counter's reading for the copy kernel to that size is the scale to apply to the same counter's reading for the
    race kernel (run this under rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE)."""
    n = mib * (1 << 20) // 4
    src = torch.arange(n, dtype=torch.int32, device=dev)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"entry": "calibrate", "copies": reps, "MiB_read_per_copy": mib, "MiB_written_per_copy": mib}),
          flush=True)
    return 0


def bench_arrival_tree(args, w, dev):
    """Algorithm 5 tree form (ersd_race_verify_arrival_tree); events bracket the whole call (five kernels)."""
    from paper_2504_15475_amd import race, workloads as wl
    base = wl.make_inputs(w, dev)
    sets = [base]
    for _ in range(max(1, args.buffers) - 1):
        sets.append(dict(base, draft=(base["draft"].float() + 0.01 * torch.randn(base["draft"].shape, device=dev))
                         .to(w.dtype).contiguous(),
                         target=(base["target"].float() + 0.01 * torch.randn(base["target"].shape, device=dev))
                         .to(w.dtype).contiguous()))
    B, C, V = base["draft"].shape
    code = race._dtype_code(base["draft"])
    ws = torch.empty(race.arrival_tree_workspace_bytes(B, C - 1, V, code), dtype=torch.uint8, device=dev)

    plan = race.arrival_tree_prepare(base["parent"], base["rank"])   # the tree does not change from step to step

    def step(i):
        x = sets[i % len(sets)]
        return race.race_verify_arrival_tree(x["draft"], x["target"], x["parent"], x["rank"], w.temperature, w.seed,
                                             workspace=ws, plan=plan)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    K = args.steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(K):
        out = step(i)
    e1.record()
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    gpu_ms = e0.elapsed_time(e1) / K
    elements = w.race_elements
    nbytes = elements * w.elem_bytes
    line = {
        "metric": "race_elements_per_sec", "value": elements * K / total_s, "unit": "elements/s", "n_gpus": 1,
        "steps": K, "warmup": args.warmup, "ms_per_step": total_s * 1e3 / K, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": ARITHMETIC, "data": "synthetic",
        "config": {"workload": w.name, "entry": "ersd_race_verify_arrival_tree", "contexts": B * C, "V": V,
                   "philox_rounds": race.philox_rounds(), "mean_accept_len": float(out[2].float().mean())},
        "roofline": {"bound": "hbm", "achieved": round(nbytes / (gpu_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(nbytes / (gpu_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None,
                     "kernel": "whole call with a prepared tree shape (races, resolve, walk)",
                     "kernel_ms_avg": round(gpu_ms, 5), "algorithmic_bytes_per_launch": nbytes},
    }
    if not args.no_cpu_baseline:
        from oracle import race_verify_arrival_tree, num_threads
        nb = min(B, 4)
        d_host, t_host = base["draft"][:nb].cpu(), base["target"][:nb].cpu()
        par, rk = base["parent"].cpu().numpy(), base["rank"].cpu().numpy()
        t1 = time.perf_counter()
        ora = race_verify_arrival_tree(d_host, t_host, par, rk, w.temperature, w.seed, max_rank=race.max_rank())
        dt = time.perf_counter() - t1
        got = race.race_verify_arrival_tree(base["draft"], base["target"], base["parent"], base["rank"], w.temperature,
                                            w.seed, workspace=ws)
        torch.cuda.synchronize()
        mism = int((got[0][:nb].cpu().numpy() != ora["draft_tokens"]).sum()
                   + (got[1][:nb].cpu().numpy() != ora["target_tokens"]).sum()
                   + (got[2][:nb].cpu().numpy() != ora["accept_len"]).sum())
        line["cpu_baseline"] = {"value": elements * nb / B / dt, "unit": "elements/s", "cores": num_threads(),
                                "kind": "oracle", "sample": f"first {nb} of {B} prompts, one pass",
                                "check": {"mismatches_vs_oracle": mism}}
    print(json.dumps(line), flush=True)
    return 0


def bench_gsd_tree(args, w, dev):
    """The comparison method on the draft tree of workload 5 (ersd_gsd_verify_tree, Algorithm 4's verification) on the
    logits and drafted tokens of the arrival-tree verification; events bracket the call (one kernel)."""
    from paper_2504_15475_amd import race, workloads as wl
    base = wl.make_inputs(w, dev)
    sets = [base]
    for _ in range(max(1, args.buffers) - 1):
        sets.append(dict(base, draft=(base["draft"].float() + 0.01 * torch.randn(base["draft"].shape, device=dev))
                         .to(w.dtype).contiguous(),
                         target=(base["target"].float() + 0.01 * torch.randn(base["target"].shape, device=dev))
                         .to(w.dtype).contiguous()))
    plan = race.arrival_tree_prepare(base["parent"], base["rank"])
    for x in sets:  # the drafting stage is not part of verification
        x["tokens"] = race.race_verify_arrival_tree(x["draft"], x["target"], x["parent"], x["rank"], w.temperature,
                                                    w.seed, plan=plan)[0]
    B, C, V = base["draft"].shape

    def step(i):
        x = sets[i % len(sets)]
        return race.gsd_verify_tree(x["draft"], x["target"], x["parent"], x["rank"], x["tokens"], w.temperature, w.seed,
                                    plan=plan)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    K = args.steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(K):
        out = step(i)
    e1.record()
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    gpu_ms = e0.elapsed_time(e1) / K
    print(json.dumps({
        "metric": "verification_steps_per_sec", "value": K / total_s, "unit": "steps/s", "n_gpus": 1,
        "steps": K, "warmup": args.warmup, "ms_per_step": total_s * 1e3 / K, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 exponentials, f64 sums and residual recursion", "data": "synthetic",
        "config": {"workload": w.name, "entry": "ersd_gsd_verify_tree (comparison method, Algorithm 4's verification)",
                   "B": B, "contexts": C, "V": V, "mean_accept_len": float(out[0].float().mean())},
        "latency": {"ms_per_call_gpu_events": round(gpu_ms, 5),
                    "note": "one workgroup per prompt walks its tree; the rows read depend on the walk"},
        "roofline": None,
    }), flush=True)
    return 0


def bench_gsd(args, w, dev):
    """The comparison method on a sequence workload's logits; events bracket the whole call (four kernels)."""
    from paper_2504_15475_amd import race, workloads as wl
    if w.variant != "sequence":
        print("bench.py: --entry gsd needs a sequence workload (0, 1 or 2)", file=sys.stderr)
        return 2
    base = wl.make_inputs(w, dev)
    sets = [base]
    for _ in range(max(1, args.buffers) - 1):
        sets.append(dict(draft=(base["draft"].float() + 0.01 * torch.randn(base["draft"].shape, device=dev))
                         .to(w.dtype).contiguous(),
                         target=(base["target"].float() + 0.01 * torch.randn(base["target"].shape, device=dev))
                         .to(w.dtype).contiguous()))
    for x in sets:  # the drafting stage is not part of verification
        x["tokens"] = race.race_sample(x["draft"].unsqueeze(1), 0, w.temperature, w.seed)[:, 0].contiguous()
    B, k, V = base["draft"].shape
    ws = torch.empty(race.gsd_workspace_bytes(B, k, V, race._dtype_code(base["draft"])), dtype=torch.uint8, device=dev)

    def step(i):
        x = sets[i % len(sets)]
        return race.gsd_verify(x["draft"], x["target"], x["tokens"], w.temperature, w.seed, workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    K = args.steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(K):
        out = step(i)
    e1.record()
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    gpu_ms = e0.elapsed_time(e1) / K
    # every drafted position's two rows once, then the two rows of the rejected position (or the last target row)
    elements = B * (2 * k + 2) * V
    nbytes = elements * w.elem_bytes
    print(json.dumps({
        "metric": "race_elements_per_sec", "value": elements * K / total_s, "unit": "elements/s", "n_gpus": 1,
        "steps": K, "warmup": args.warmup, "ms_per_step": total_s * 1e3 / K, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32 normalisers and weights, f64 where f32 cannot decide", "data": "synthetic",
        "config": {"workload": w.name, "entry": "ersd_gsd_verify (comparison method)", "B": B, "k": k, "V": V,
                   "mean_accept_len": float(out[0].float().mean())},
        "roofline": {"bound": "hbm", "achieved": round(nbytes / (gpu_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(nbytes / (gpu_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None,
                     "kernel": "whole call (normalisers, accept, residual, pick)", "kernel_ms_avg": round(gpu_ms, 5),
                     "algorithmic_bytes_per_launch": nbytes},
    }), flush=True)
    return 0


def bench_sample(args, w, dev):
    """One-model races (ersd_race_sample).  --npos 0: all target rows of the workload in one call (what verification
    with separate draft and target calls does).  --npos 1: the drafting call of Algorithm 2, one position of every
    sequence per call (B x 1 x V), k calls per step, on the workload's draft logits; this call is bound by latency,
    not bandwidth, and is reported in microseconds per call."""
    from paper_2504_15475_amd import race, workloads as wl
    inputs = wl.make_inputs(w, dev)
    K = args.steps
    if args.npos == 1:
        if w.variant == "tree":
            print("bench.py: --npos 1 needs a sequence or multi-draft workload", file=sys.stderr)
            return 2
        d = inputs["draft"] if w.variant == "multi" else inputs["draft"].unsqueeze(1)      # [B, m, k, V]
        B, m, k, V = d.shape
        calls = []
        for s_ in range(max(1, args.buffers)):
            src = d if s_ == 0 else (d.float() + 0.01 * torch.randn(d.shape, device=dev)).to(d.dtype)
            calls.append([race.PreparedSample(src[:, :, j:j + 1].contiguous(), j, w.temperature, w.seed)
                          for j in range(k)])
        del d, inputs
        for i in range(args.warmup):
            for c in calls[i % len(calls)]:
                c.run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(K):
            for c in calls[i % len(calls)]:
                c.run()
        e1.record()
        torch.cuda.synchronize()
        total_s = time.perf_counter() - t0
        ncalls = K * k
        gpu_us = e0.elapsed_time(e1) * 1e3 / ncalls
        elements = B * m * V
        nbytes = elements * calls[0][0].x.element_size()
        print(json.dumps({
            "metric": "race_elements_per_sec", "value": elements * ncalls / total_s, "unit": "elements/s", "n_gpus": 1,
            "steps": K, "warmup": args.warmup, "ms_per_step": total_s * 1e3 / K, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": ARITHMETIC, "data": "synthetic",
            "config": {"workload": w.name + ":draft rows, one position per call", "entry": "ersd_race_sample",
                       "rows_per_call": B * m, "V": V, "calls_per_step": k, "bytes_per_call": nbytes,
                       "philox_rounds": race.philox_rounds()},
            "latency": {"us_per_call_gpu_events": round(gpu_us, 3), "us_per_call_wall": round(total_s * 1e6 / ncalls, 3),
                        "calls_timed": ncalls,
                        "note": "events around all calls, issued back to back; two kernels per call (race, resolve)"},
            "roofline": {"bound": "hbm", "achieved": round(nbytes / (gpu_us * 1e-6) / 1e9, 1), "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": round(nbytes / (gpu_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None,
                         "kernel": "race_kernel + resolve_kernel (whole call)", "kernel_ms_avg": round(gpu_us * 1e-3, 6),
                         "algorithmic_bytes_per_launch": nbytes},
        }), flush=True)
        return 0

    base = inputs["target"]
    if w.variant != "multi":
        base = base.unsqueeze(1)
    base = base.contiguous()
    sets = [base] + [(base.float() + 0.01 * torch.randn(base.shape, device=dev)).to(base.dtype).contiguous()
                     for _ in range(max(1, args.buffers) - 1)]
    B, m, npos, V = base.shape
    calls = [race.PreparedSample(x, 0, w.temperature, w.seed) for x in sets]
    for i in range(args.warmup):
        calls[i % len(calls)].run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(K):
        calls[i % len(calls)].run()
    e1.record()
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    elements = base.numel()
    gpu_ms = e0.elapsed_time(e1) / K
    nbytes = elements * base.element_size()
    print(json.dumps({
        "metric": "race_elements_per_sec", "value": elements * K / total_s, "unit": "elements/s", "n_gpus": 1,
        "steps": K, "warmup": args.warmup, "ms_per_step": total_s * 1e3 / K, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": ARITHMETIC, "data": "synthetic",
        "config": {"workload": w.name + ":target rows only", "entry": "ersd_race_sample", "rows": B * m * npos, "V": V,
                   "philox_rounds": race.philox_rounds()},
        "roofline": {"bound": "hbm", "achieved": round(nbytes / (gpu_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(nbytes / (gpu_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None,
                     "kernel": "race_kernel + resolve_kernel (whole call)", "kernel_ms_avg": round(gpu_ms, 5),
                     "algorithmic_bytes_per_launch": nbytes},
    }), flush=True)
    return 0


def oracle_side(w, base, call, variant, timed):
    """The CPU oracle on a bounded sample of the same inputs.  Always: its tokens and accept lengths against the GPU's
    on that sample.  With `timed`: the oracle, as it stands, run for roughly 15 s of CPU work on this machine's host cores
    (the reported CPU baseline)."""
    import numpy as np
    import oracle
    from paper_2504_15475_amd import race
    # sample: leading sequences; about 20 ns per token position and core on this class of host
    per_seq_positions = (w.m * (w.k + 1) if w.variant != "tree" else w.N) * w.V
    nseq = max(1, min(w.B, int((3.0e8 if timed else 1.0e8) // per_seq_positions)))
    d = base["draft"][:nseq].contiguous().cpu()
    t = base["target"][:nseq].contiguous().cpu()
    oracle.race_rows(None, t.reshape(-1, w.V)[0], w.temperature, w.seed)  # warm-up (library load, page-in)
    passes = max(1, min(50, int(7.5e8 // (per_seq_positions * nseq)))) if timed else 1
    t0 = time.perf_counter()
    for _ in range(passes):
        if variant == race.VARIANT_SEQUENCE:
            o = oracle.race_verify(d, t, w.temperature, w.seed, want_info=True)
        elif variant == race.VARIANT_MULTI:
            o = oracle.race_verify_multi(d, t, w.temperature, w.seed, want_info=True)
        else:
            o = oracle.race_verify_tree(d, t, base["parent"].cpu().numpy(), w.temperature, w.seed, want_info=True)
    dt = time.perf_counter() - t0
    elements = w.race_elements * nseq // w.B * passes
    call.run()
    torch.cuda.synchronize()
    gpu = [x.cpu().numpy() for x in call.outputs()]
    mism = int((gpu[0][:nseq] != o["draft_tokens"]).sum() + (gpu[1][:nseq] != o["target_tokens"]).sum())
    mism_acc = int((gpu[2][:nseq] != o["accept_len"]).sum())
    near = int(o["draft_info"]["near_tie"].sum() + o["target_info"]["near_tie"].sum())
    check = {"sample_sequences": nseq, "of": w.B, "token_mismatches_vs_oracle": mism,
             "accept_len_mismatches_vs_oracle": mism_acc, "oracle_near_tie_rows": near,
             "mean_accept_len_gpu": float(np.mean(gpu[2]))}
    if not timed:
        return None, check
    base_out = {"value": elements / dt, "unit": "elements/s", "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"first {nseq} of {w.B} sequences of the same workload, {passes} passes, {elements} race "
                          f"elements, {dt:.2f} s wall on {oracle.num_threads()} threads"}
    return base_out, check


if __name__ == "__main__":
    sys.exit(main())
