#!/usr/bin/env python3
"""Throughput of the exponential-race verification hot path on one MI355X.

One "step" is one pass of the whole hot path (race kernel + acceptance kernel) over one batch of synthetic
logits that are already resident in HBM.  The default workload is the B=64, k=8, V=128256 bf16 sequence
configuration the headline metric is quoted on.  Prints ONE JSON line.

The step is issued as its two stages (ersd_race_stage_races, ersd_race_stage_accept -- together exactly
ersd_race_verify*) so that a HIP event can be recorded between them: the race kernel's own duration is
measured inside the timed region and priced against the HBM roofline.  Input buffers rotate over several
distinct sets so that the 256 MB on-die cache cannot serve the reads.
"""
import argparse
import json
import os
import sys
import time

import torch

PEAK_HBM_GBS = 8000.0

# HBM bytes per race-kernel launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by a copy
# kernel of known size; filled in from the summaries under profiles/ (None = not measured for that workload).
MEASURED_TRAFFIC_BYTES = {1: 286262270, 2: 5171172134, 3: 1118971385, 4: 1068091931}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=1,
                    help="index into the five benchmark workloads (default 1); 5 = the tree of workload 4 verified "
                         "as Algorithm 5 states it (children of a context = first arrivals of one race)")
    ap.add_argument("--buffers", type=int, default=4, help="distinct input sets rotated through (cache defeat)")
    ap.add_argument("--event-every", type=int, default=8,
                    help="record HIP events around the race kernel of every N-th timed step (events cost a few us)")
    ap.add_argument("--entry", choices=["verify", "sample", "gsd"], default="verify",
                    help="verify: the fused draft+target races (default, the headline metric); sample: the one-model "
                         "entry point on the workload's target logits (how a serving loop calls the race); gsd: the "
                         "comparison method (ersd_gsd_verify) on the same logits, sequence workloads only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fused-call", action="store_true",
                    help="issue each step through the single verify entry point (no event between the stages)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus must be 1",
              file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        return 2

    from paper_2504_15475_amd import race, workloads as wl
    race.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == 5:
        return bench_arrival_tree(args, wl.ARRIVAL_TREE, dev)
    w = wl.WORKLOADS[args.workload]
    variant = {"sequence": race.VARIANT_SEQUENCE, "multi": race.VARIANT_MULTI, "tree": race.VARIANT_TREE}[w.variant]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.entry == "sample":
        return bench_sample(args, w, dev)
    if args.entry == "gsd":
        return bench_gsd(args, w, dev)

    base = wl.make_inputs(w, dev)
    sets = [base]
    for i in range(1, max(1, args.buffers)):
        # further sets: same distribution, different values (a cheap permutation of rows would alias in cache)
        g = torch.Generator(device=dev).manual_seed(5000 + i)
        noise = lambda x: (x.float() + 0.01 * torch.randn(x.shape, generator=g, device=dev)).to(x.dtype).contiguous()
        s = dict(draft=noise(base["draft"]), target=noise(base["target"]))
        if "parent" in base:
            s["parent"] = base["parent"]
        sets.append(s)
    calls = [race.PreparedVerify(variant, s["draft"], s["target"], w.temperature, w.seed, s.get("parent")) for s in sets]
    torch.cuda.synchronize()

    def step(i, mid=None):
        c = calls[i % len(calls)]
        if args.fused_call:
            c.run()
        else:
            c.run_stages(mid)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    K = args.steps
    every = max(1, args.event_every)
    sampled = [] if args.fused_call else [i for i in range(K) if i % every == every - 1 or K < every]
    ev0 = {i: torch.cuda.Event(enable_timing=True) for i in sampled}
    ev1 = {i: torch.cuda.Event(enable_timing=True) for i in sampled}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        if i in ev0:
            ev0[i].record()
            step(i, ev1[i])
        else:
            step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    total_s = t1 - t0
    ms_per_step = total_s * 1e3 / K
    value = w.race_elements * K / total_s
    if args.fused_call:
        kernel_ms = None
    else:
        durs = sorted(ev0[i].elapsed_time(ev1[i]) for i in sampled)
        kernel_ms = sum(durs) / len(durs)
    algo_bytes = w.logit_bytes
    roofline = None
    if kernel_ms:
        achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(w.index),
                    "kernel": "race_kernel", "launches_timed": len(durs), "kernel_ms_avg": round(kernel_ms, 5),
                    "kernel_ms_min": round(durs[0], 5), "kernel_ms_median": round(durs[len(durs) // 2], 5),
                    "algorithmic_bytes_per_launch": algo_bytes}

    if roofline is not None:
        # context, outside the timed region: the same tensors read once by a kernel that does nothing else, with the
        # race kernel's loads and launch shape
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        n_probe = 24
        pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_probe)]
        for i in range(4):
            race.read_probe(sets[i % len(sets)]["draft"], sets[i % len(sets)]["target"], sink)
        for i, (e0, e1) in enumerate(pe):
            e0.record()
            race.read_probe(sets[i % len(sets)]["draft"], sets[i % len(sets)]["target"], sink)
            e1.record()
        torch.cuda.synchronize()
        probe_ms = sum(e0.elapsed_time(e1) for e0, e1 in pe) / n_probe
        roofline["plain_read_same_shape"] = {"ms": round(probe_ms, 5),
                                             "GB/s": round(algo_bytes / (probe_ms * 1e-3) / 1e9, 1),
                                             "race_kernel_vs_plain_read": round(probe_ms / kernel_ms, 4)}

    out = {
        "metric": "race_elements_per_sec", "value": value, "unit": "elements/s", "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": w.name, "description": wl.describe(w), "race_elements_per_step": w.race_elements,
                   "logit_dtype": "bf16" if w.elem_bytes == 2 else "fp32", "input_buffer_sets": len(calls),
                   "arithmetic": "u32 Philox + f32 bound filter on every token, f64 scores where f32 cannot decide",
                   "philox_rounds": race.philox_rounds(),
                   "issue": "verify entry point" if args.fused_call else "two stage entry points + event"},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["check"] = cpu_baseline(w, base, calls[0], variant)
    print(json.dumps(out), flush=True)
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

    def step(i):
        x = sets[i % len(sets)]
        return race.race_verify_arrival_tree(x["draft"], x["target"], x["parent"], x["rank"], w.temperature, w.seed,
                                             workspace=ws)

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
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": w.name, "entry": "ersd_race_verify_arrival_tree", "contexts": B * C, "V": V,
                   "philox_rounds": race.philox_rounds(), "mean_accept_len": float(out[2].float().mean())},
        "roofline": {"bound": "hbm", "achieved": round(nbytes / (gpu_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(nbytes / (gpu_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None,
                     "kernel": "whole call (tree shape, races, two resolve kernels, walk)",
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
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "entry": "ersd_gsd_verify (comparison method)", "B": B, "k": k, "V": V,
                   "mean_accept_len": float(out[0].float().mean())},
        "roofline": {"bound": "hbm", "achieved": round(nbytes / (gpu_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(nbytes / (gpu_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None,
                     "kernel": "whole call (normalisers, accept, residual, pick)", "kernel_ms_avg": round(gpu_ms, 5),
                     "algorithmic_bytes_per_launch": nbytes},
    }), flush=True)
    return 0


def bench_sample(args, w, dev):
    """One-model races (ersd_race_sample) on the workload's target logits; events bracket the whole call."""
    from paper_2504_15475_amd import race, workloads as wl
    base = wl.make_inputs(w, dev)["target"]
    if w.variant != "multi":
        base = base.unsqueeze(1)
    base = base.contiguous()
    sets = [base] + [(base.float() + 0.01 * torch.randn(base.shape, device=dev)).to(base.dtype).contiguous()
                     for _ in range(max(1, args.buffers) - 1)]
    B, m, npos, V = base.shape
    need = int(race.lib().ersd_race_sample_workspace_bytes(B, m, npos, V, race._dtype_code(base)))
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    for i in range(args.warmup):
        race.race_sample(sets[i % len(sets)], 0, w.temperature, w.seed, workspace=ws)
    torch.cuda.synchronize()
    K = args.steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(K):
        race.race_sample(sets[i % len(sets)], 0, w.temperature, w.seed, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    elements = base.numel()
    gpu_ms = e0.elapsed_time(e1) / K
    nbytes = elements * base.element_size()
    print(json.dumps({
        "metric": "race_elements_per_sec", "value": elements * K / total_s, "unit": "elements/s", "n_gpus": 1,
        "steps": K, "warmup": args.warmup, "ms_per_step": total_s * 1e3 / K, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": w.name + ":target rows only", "entry": "ersd_race_sample", "rows": B * m * npos, "V": V,
                   "philox_rounds": race.philox_rounds()},
        "roofline": {"bound": "hbm", "achieved": round(nbytes / (gpu_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(nbytes / (gpu_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": None,
                     "kernel": "race_kernel + resolve_kernel (whole call)", "kernel_ms_avg": round(gpu_ms, 5),
                     "algorithmic_bytes_per_launch": nbytes},
    }), flush=True)
    return 0


def cpu_baseline(w, base, call, variant):
    """The CPU oracle, as it stands, on a bounded sample of the same inputs, timed on this machine's host cores; its
    tokens are also compared with the GPU's on that sample."""
    import numpy as np
    import oracle
    from paper_2504_15475_amd import race
    # sample: leading sequences, repeated so that the oracle does roughly 15 s of CPU work (about 20 ns per token
    # position and core on this class of host)
    per_seq_positions = (w.m * (w.k + 1) if w.variant != "tree" else w.N) * w.V
    nseq = max(1, min(w.B, int(3.0e8 // per_seq_positions)))
    d = base["draft"][:nseq].contiguous().cpu()
    t = base["target"][:nseq].contiguous().cpu()
    oracle.race_rows(None, t.reshape(-1, w.V)[0], w.temperature, w.seed)  # warm-up (library load, page-in)
    passes = max(1, min(50, int(7.5e8 // (per_seq_positions * nseq))))
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
    base_out = {"value": elements / dt, "unit": "elements/s", "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"first {nseq} of {w.B} sequences of the same workload, {passes} passes, {elements} race "
                          f"elements, {dt:.2f} s wall on {oracle.num_threads()} threads"}
    check = {"sample_sequences": nseq, "token_mismatches_vs_oracle": mism, "accept_len_mismatches_vs_oracle": mism_acc,
             "oracle_near_tie_rows": near, "mean_accept_len_gpu": float(np.mean(gpu[2]))}
    return base_out, check


if __name__ == "__main__":
    sys.exit(main())
