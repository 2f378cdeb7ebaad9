#!/usr/bin/env python3
"""Benchmark of the transfer-tuning hot path on one MI355X.

A step is one network-shaped pass over the workload's fused kernels, each under the best
TRANSFERRED schedule (the fastest valid donor record of its class, or the default as fallback),
with all inputs resident in HBM and every launch of the pass on tensors of its own (a network's
layers do not share weights or activations; the pass touches far more than the caches hold, so
every launch finds its operands cold).  `value` is the pass's algorithmic FLOPs over its time; the
time of the same launches repeated on one set of tensors per kernel is reported beside it as the
cache-warm figure.  The same run re-times, per kernel, the record an exhaustive native sweep found
and reports the transferred schedule's speed as a fraction of it.

The sweeps are the search, not the step.  The records the timed pass uses are the stored outcome of
`--sweep` (tuned/<workload>.json, with the donor pool in tuned/<workload>.pool), the same records
the parity tests check.  After the timed region the default run repeats the transfer sweep and the
native sweep live, so their pair counts and wall-clock (the paper's "search time") are measured in
this run; `--no-live-sweep` leaves that out (used for profiles, so that a kernel trace of the
command holds the launches of the pass and of the per-kernel timing only).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--sweep] [--no-live-sweep]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"hbm": 8000.0, "mfma_bf16": 2500.0, "mfma_f32": 157.3}  # GB/s, TFLOP/s (dense, published)


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "seq128_from_256",
                                                           "seq256_from_128"])
    ap.add_argument("--sweep", action="store_true", help="run the sweeps and store their outcome")
    ap.add_argument("--retune-pool", action="store_true", help="also re-tune the donor kernels (the pool)")
    ap.add_argument("--donor-limit", type=int, default=0, help="use only the first N donor kernels")
    ap.add_argument("--pool-only", action="store_true", help="with --retune-pool: stop once the pool file is written")
    ap.add_argument("--resume-pool", default="", help="pool checkpoint of an interrupted --retune-pool run to continue from")
    ap.add_argument("--level", type=int, default=1, help="size of the enumerated native space (0, 1, 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-live-sweep", action="store_true", help="do not repeat the sweeps after the timed region")
    ap.add_argument("--sweep-cold-mb", type=int, default=600,
                    help="megabytes of tensor sets the sweeps' launches rotate through (0: one set, cache-warm timing)")
    ap.add_argument("--sweep-cold-min-mb", type=int, default=32,
                    help="kernels whose tensors take less than this are timed on one tensor set in the sweeps")
    ap.add_argument("--kernels", default="", help="comma-separated kernel names: restrict the workload to them")
    ap.add_argument("--cold-mb", type=int, default=600,
                    help="per-kernel timing rotates over tensor sets of at least this many MB in total")
    ap.add_argument("--chain", action="store_true",
                    help="cfg5 only: time the bottleneck blocks wired output-to-input against the same launches on "
                         "independent tensors and against the sum of standalone times (prints its own JSON line)")
    return ap.parse_args()


def knobs_to_record(api, knobs):
    return None if knobs is None else api.make_schedule(**knobs)


def run_sweeps(args, api, tune, wl, targets, dks, donors, cfg, tuned_path, pool_path):
    """Donor tuning (if needed), transfer sweep and native sweep of the targets; writes the tuned file."""
    import torch
    t_all = time.time()
    if args.retune_pool or not os.path.exists(pool_path):
        if args.donor_limit:
            donors = donors[:args.donor_limit]
        log(f"[pool] native-tuning {len(donors)} donor kernels")
        t0 = time.time()
        per_donor = 4 if args.workload == "cfg1" else 1
        partial = os.path.join(ROOT, "gpurun_out", f"{args.workload}.pool.partial")
        pool = tune.tune_donors(donors, cfg + 100, args.level, log, per_donor,
                                partial if os.path.isdir(os.path.dirname(partial)) else None, args.resume_pool or None,
                                cold_mb=args.sweep_cold_mb, cold_min_mb=args.sweep_cold_min_mb)
        tune.save_pool(pool_path, pool, [donors[i // per_donor].name for i in range(len(pool))])
        pool_seconds = time.time() - t0
        mirror = os.path.join(ROOT, "gpurun_out", "tuned")
        if os.path.isdir(os.path.dirname(mirror)):
            import shutil
            os.makedirs(mirror, exist_ok=True)
            shutil.copy(pool_path, os.path.join(mirror, os.path.basename(pool_path)))
        if args.pool_only:
            log(f"[pool] {len(pool)} records in {pool_seconds:.0f}s; stopping as asked")
            sys.exit(0)
    else:
        pool = tune.load_pool(pool_path)
        pool_seconds = None
    log(f"[sweep] transfer sweep: {len(dks)} kernels x {len(pool)} records")
    rows, table, evals, wall = api.tt_transfer_sweep(dks, pool, api.make_opts(**tune.FULL))
    out = dict(workload=args.workload, pool_records=len(pool), pool_seconds=pool_seconds,
               sweep_timing=f"kernels of at least {args.sweep_cold_min_mb} MB: every launch of a pair on the next of enough "
                            f"tensor sets to hold {args.sweep_cold_mb} MB; smaller kernels on one tensor set"
               if args.sweep_cold_mb else "all launches of a pair on one tensor set (cache-warm)", transfer_pairs=evals,
               transfer_wall_seconds=wall, kernels=[])
    n_invalid = sum(r["n_invalid"] for r in rows)
    out["transfer_invalid_pairs"] = n_invalid
    log(f"[sweep] {evals} pairs in {wall:.1f}s, {n_invalid} invalid")
    t0 = time.time()
    for k, dk, r in zip(targets, dks, rows):
        best, best_us, default_us, n_valid, n_rec = tune.native_sweep(dk, args.level)
        chosen = pool[r["chosen"]] if r["chosen"] >= 0 else None
        out["kernels"].append(dict(
            name=k.name, cls=k.cls, chosen_pool_index=r["chosen"],
            transfer=None if chosen is None else chosen.knobs(), transfer_us=r["best_us"], default_us=r["default_us"],
            n_valid=r["n_valid"], n_invalid=r["n_invalid"],
            native=None if best is None else best.knobs(), native_us=best_us, native_valid=n_valid, native_space=n_rec))
        log(f"[native] {k.name:34s} transfer {r['best_us']:9.2f} us  native {best_us:9.2f} us  default "
            f"{r['default_us']:9.2f} us  ratio {best_us / r['best_us']:.3f}  ({n_valid}/{n_rec} valid)")
    out["native_wall_seconds"] = time.time() - t0
    out["total_seconds"] = time.time() - t_all
    tune.save_json(tuned_path, out)
    # a second copy where a remote run's outputs are collected, so the outcome can be committed
    mirror = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(mirror):
        import shutil
        os.makedirs(os.path.join(mirror, "tuned"), exist_ok=True)
        for p in (tuned_path, pool_path):
            shutil.copy(p, os.path.join(mirror, "tuned", os.path.basename(p)))
    torch.cuda.synchronize()
    return out


def chain_leg(args, api, harness, tune, wl, targets, dks, transfer):
    """Inter-kernel effects (paper Section 5.5): the bottleneck blocks 2..n of every ResNet-50 stage, chained."""
    import torch
    by_name = {k.name: i for i, k in enumerate(targets)}
    chained, records, independent, standalone_us = [], [], [], 0.0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def single(i):
        """The kernel on its private tensors, one launch per list entry."""
        return api.DeviceKernel(targets[i].cls, targets[i].shape, dks[i].tensors, 1, targets[i].name, dks[i].ws.numel())

    def standalone(i):
        one = api.KernelList([single(i)], [transfer[i]])
        one.run(3)
        e0.record()
        one.run(20)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / 20

    for st, (wd, nb) in enumerate(zip([64, 128, 256, 512], [3, 4, 6, 3]), start=1):
        cout = wd * 4
        ir = by_name[f"r50_s{st}_reduce_{cout}_{wd}"]
        ic = by_name["r50_s1_b1_3x3_s1" if st == 1 else f"r50_s{st}_3x3"]
        ie = by_name[f"r50_s{st}_expand_{wd}_{cout}_res"]
        blocks = nb - 1
        cd, _, _ = harness.bottleneck_chain(targets[ir], targets[ic], targets[ie], blocks, wl.seed_for(5, 900 + st))
        chained += cd
        records += [transfer[ir], transfer[ic], transfer[ie]] * blocks
        us = [standalone(i) for i in (ir, ic, ie)]
        standalone_us += blocks * sum(us)
        independent += [single(i) for _ in range(blocks) for i in (ir, ic, ie)]

    def timed(klist):
        klist.run(args.warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        klist.run(args.steps)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / args.steps

    chain_us = timed(api.KernelList(chained, records))
    indep_us = timed(api.KernelList(independent, records))
    flops = sum(d_k.flops() for d_k in [targets[by_name[d.name.split("@")[0]]] for d in chained])
    print(json.dumps({"chain": {"launches": len(chained), "gflop": flops / 1e9, "chained_us": chain_us,
                                "same_launches_on_independent_tensors_us": indep_us,
                                "sum_of_standalone_us": standalone_us,
                                "chained_over_standalone": chain_us / standalone_us}}))


def machine_rates(api):
    """What plain kernels reach on this GPU (tt_debug_probe), to set beside the roofline fractions."""
    import torch
    n = 768 << 20                                    # per buffer: a copy streams 1.5 GB, six times the memory-side cache
    src = torch.ones(n // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    small = torch.ones((2 << 20) // 4, dtype=torch.int32, device="cuda")
    r = dict(
        launch_gap_us=api.tt_debug_probe(api.TT_PROBE_LAUNCH_GAP_US, reps=200),
        mfma_bf16_tflops=api.tt_debug_probe(api.TT_PROBE_MFMA_BF16_TFLOPS, dst=small, reps=5),
        copy_linear_cold_gbps=api.tt_debug_probe(api.TT_PROBE_COPY_LINEAR_GBPS, src, dst, reps=4),
        copy_tiled_cold_gbps=api.tt_debug_probe(api.TT_PROBE_COPY_TILED_GBPS, src, dst, reps=4),
        l2_read_gbps=api.tt_debug_probe(api.TT_PROBE_L2_READ_GBPS, small, dst, reps=5),
        what="plain kernels of the library timed like the operators: empty launches back to back; 32x32x16 bf16 MFMA "
             "only; read+write rate of a 768 MiB copy, linear and in 64-row x 128-byte tiles of 512-byte rows; reads "
             "of a 2 MiB source by all CUs")
    del src, dst, small
    torch.cuda.empty_cache()
    return r


def cpu_baseline_leg(wl, targets, budget_s=25.0):
    """The oracle, as it stands, on the host cores: each distinct kernel of the workload once, largest first,
    until the time budget is spent."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from oracle import ops as O
    import parity
    cores = O.max_threads()
    flops = secs = 0.0
    used = 0
    for i in sorted(range(len(targets)), key=lambda i: -targets[i].flops()):
        k = targets[i]
        inp = wl.make_inputs(k, 99 + i)
        t0 = time.perf_counter()
        parity.oracle_output(k, inp)
        secs += time.perf_counter() - t0
        flops += k.flops()
        used += 1
        if secs > budget_s:
            break
    return dict(value=flops / secs / 1e12, unit="TFLOP/s", cores=cores, kind="oracle",
                sample=f"oracle (naive C loops, fp64 accumulate, OpenMP over the outermost output axis) on the {used} "
                       f"largest of {len(targets)} kernels at full size, one launch each: {flops / 1e9:.1f} GFLOP in "
                       f"{secs:.1f} s")


def clone_kernel(api, k, dk, use_count=1):
    """The same kernel on fresh copies of its activations, residual and output (weights and bias too: a
    network's layers do not share them)."""
    tensors = {name: t.clone() for name, t in dk.tensors.items()}
    return api.DeviceKernel(k.cls, k.shape, tensors, use_count, k.name, dk.ws.numel())


def live_sweeps(args, api, tune, targets, dks, pool, by_name):
    """The search, measured in this run: transfer sweep over the whole pool, native sweep of every target,
    and the cheaper variants (pair budget, priority, local refinement)."""
    t0 = time.time()
    rows, table, evals, wall = api.tt_transfer_sweep(dks, pool, api.make_opts(**tune.FULL))
    same = sum(1 for k, r in zip(targets, rows) if r["chosen"] == by_name[k.name]["chosen_pool_index"])
    total_us = sum(r["best_us"] * k.use_count for k, r in zip(targets, rows))
    default_total_us = sum(r["default_us"] * k.use_count for k, r in zip(targets, rows))
    out = dict(swept_in_this_run=True, pairs=evals, wall_seconds=wall,
               invalid_pairs=sum(r["n_invalid"] for r in rows), pool_records=len(pool),
               kernels_on_default_fallback=sum(1 for r in rows if r["chosen"] < 0),
               kernels_with_the_stored_choice=same, pass_us_by_standalone_times=total_us,
               untuned_pass_us_by_standalone_times=default_total_us)
    log(f"[live] transfer sweep: {evals} pairs in {wall:.2f}s, {out['invalid_pairs']} invalid, "
        f"{out['kernels_on_default_fallback']} kernels on the default, {same}/{len(targets)} choices as stored")
    # cheaper sweeps: a quarter of the donor evaluations, sampled uniformly / spent by share of untuned time
    donor_pairs = evals - len(dks)
    cheaper = {}
    for name, prio in (("uniform_quarter", 0), ("priority_quarter", 1)):
        r2, _, e2, w2 = api.tt_transfer_sweep(dks, pool, api.make_opts(pair_budget=max(1, donor_pairs // 4),
                                                                       prioritise=prio, seed=2022, **tune.FULL))
        us2 = sum(r["best_us"] * k.use_count for k, r in zip(targets, r2))
        cheaper[name] = dict(pairs=e2, wall_seconds=w2, pass_us_by_standalone_times=us2,
                             speed_vs_full_sweep=total_us / us2)
        log(f"[live] {name}: {e2} pairs in {w2:.2f}s, pass {us2:.1f} us vs {total_us:.1f} us with the full sweep")
    # local refinement of the transferred record, one round
    t1 = time.time()
    refined_us, tried = 0.0, 0
    for k, dk, r in zip(targets, dks, rows):
        base = pool[r["chosen"]] if r["chosen"] >= 0 else api.tt_schedule_default(k.cls, k.shape)
        rc, best, best_us, base_us, n = api.tt_refine(dk, base, 1, api.make_opts(**tune.FULL))
        refined_us += (best_us if rc == api.TT_OK else r["best_us"]) * k.use_count
        tried += n
    cheaper["refine_one_round"] = dict(pairs=tried, wall_seconds=time.time() - t1,
                                       pass_us_by_standalone_times=refined_us, speed_vs_full_sweep=total_us / refined_us)
    log(f"[live] refinement: {tried} pairs in {time.time() - t1:.2f}s, pass {refined_us:.1f} us")
    out["cheaper_sweeps"] = cheaper
    # the native (exhaustive) sweep of every target: the denominator of "% of the native optimum"
    t2 = time.time()
    ratios = []
    for k, dk, r in zip(targets, dks, rows):
        best, best_us, default_us, n_valid, n_rec = tune.native_sweep(dk, args.level)
        ratios.append(min(best_us, r["best_us"]) / r["best_us"])
    out["native_wall_seconds"] = time.time() - t2
    out["pct_of_native_optimum_by_sweep_times"] = dict(mean=100.0 * sum(ratios) / len(ratios), min=100.0 * min(ratios),
                                                       kernels_at_or_above_80pct=sum(x >= 0.8 for x in ratios))
    out["total_seconds"] = time.time() - t0
    log(f"[live] native sweep of {len(targets)} kernels in {out['native_wall_seconds']:.1f}s; transferred vs native: "
        f"mean {out['pct_of_native_optimum_by_sweep_times']['mean']:.1f} %, min {out['pct_of_native_optimum_by_sweep_times']['min']:.1f} %")
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(kernel/schedule pairs are independent and would shard by target kernel)")
        sys.exit(2)
    import torch
    from paper_2201_05587_amd import api, harness, traffic, tune
    from paper_2201_05587_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU; there is no CPU fallback"
    torch.cuda.set_device(0)
    cfg, targets, donors = tune.workload(args.workload)
    tuned_dir = os.path.join(ROOT, "paper_2201_05587_amd", "tuned")
    os.makedirs(tuned_dir, exist_ok=True)
    tuned_path = os.path.join(tuned_dir, f"{args.workload}.json")
    pool_path = os.path.join(tuned_dir, f"{args.workload}.pool")

    seeds = [wl.seed_for(cfg, i) for i in range(len(targets))]
    if args.kernels:
        keep = [i for i, k in enumerate(targets) if k.name in args.kernels.split(",")]
        assert keep and not args.sweep, "--kernels names no kernel of the workload (and cannot be combined with --sweep)"
        targets, seeds = [targets[i] for i in keep], [seeds[i] for i in keep]
    dks = [harness.device_kernel(k, sd, max_split=8, cold_mb=args.sweep_cold_mb, cold_min_mb=args.sweep_cold_min_mb) for k, sd in zip(targets, seeds)]
    if args.sweep or not os.path.exists(tuned_path):
        tuned = run_sweeps(args, api, tune, wl, targets, dks, donors, cfg, tuned_path, pool_path)
        swept_here = True
    else:
        with open(tuned_path) as f:
            tuned = json.load(f)
        swept_here = False
    by_name = {e["name"]: e for e in tuned["kernels"]}
    transfer = [knobs_to_record(api, by_name[k.name]["transfer"]) for k in targets]
    native = [knobs_to_record(api, by_name[k.name]["native"]) for k in targets]

    if args.chain:
        assert args.workload == "cfg5", "--chain is defined for the ResNet-50-shaped configuration"
        chain_leg(args, api, harness, tune, wl, targets, dks, transfer)
        return

    # ---- timed region: K network-shaped passes under the transferred schedules, every launch on tensors
    # of its own (kernel i's use_count launches included), in network order of the kernel list ----
    launch_dks, launch_recs = [], []
    for k, dk, tr in zip(targets, dks, transfer):
        for u in range(k.use_count):
            launch_dks.append(api.DeviceKernel(k.cls, k.shape, dk.tensors, 1, k.name, dk.ws.numel()) if u == 0
                              else clone_kernel(api, k, dk))
            launch_recs.append(tr)
    cold_list = api.KernelList(launch_dks, launch_recs)
    pass_flops = sum(k.flops() * k.use_count for k in targets)
    pass_bytes = sum(k.algorithmic_bytes() * k.use_count for k in targets)
    cold_list.run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    cold_list.run(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    value = pass_flops / (elapsed / args.steps) / 1e12
    # the same launches with each kernel's use_count launches repeated on ONE set of tensors (cache-warm)
    warm_steps = max(3, args.steps // 5)
    warm_list = api.KernelList(dks, transfer)
    warm_list.run(2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    warm_list.run(warm_steps)
    torch.cuda.synchronize()
    warm_ms = (time.perf_counter() - t0) * 1e3 / warm_steps
    del cold_list, launch_dks
    torch.cuda.empty_cache()

    # ---- per-kernel durations with HIP events on the launch stream, cold: a kernel is launched in turn on
    # enough tensor sets that a set has left the caches (256 MB memory-side cache, 32 MB of L2) before its
    # turn comes again.  Every launch this process makes is entered in a ledger per kernel symbol, so the
    # average duration reported for the dominant symbol is the one a kernel trace of this same command
    # (with --no-live-sweep) shows.
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ledger = {}

    def symbol_of(k, rec):
        rec = rec if rec is not None else api.tt_schedule_default(k.cls, k.shape)
        return api.variant_name(api.tt_schedule_apply(rec, k.cls, k.shape), k.shape)

    def book(k, rec, launches, us):
        g = ledger.setdefault(symbol_of(k, rec), dict(us=0.0, flops=0.0, bytes=0.0, launches=0, dtype=k.shape.dtype,
                                                      layers=set()))
        g["us"] += us * launches
        g["flops"] += k.flops() * launches
        g["bytes"] += k.algorithmic_bytes() * launches
        g["launches"] += launches
        g["layers"].add(k.name)

    def cold_launches(k, sets, rec, rounds=3):
        """Average duration of a launch of (kernel, record) over `rounds` turns through the tensor sets."""
        ring = api.KernelList(sets, [rec] * len(sets))
        ring.run(1)
        e0.record()
        ring.run(rounds)
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (rounds * len(sets))
        book(k, rec, (rounds + 1) * len(sets), us)
        return us

    per_kernel = []
    for k, dk, tr, na in zip(targets, dks, transfer, native):
        n_sets = int(min(400, max(2, -(-args.cold_mb * 1e6 // k.algorithmic_bytes()) + 1)))
        sets = [api.DeviceKernel(k.cls, k.shape, dk.tensors, 1, k.name, dk.ws.numel())]
        sets += [clone_kernel(api, k, dk) for _ in range(n_sets - 1)]
        t_us = cold_launches(k, sets, tr)
        book(k, tr, (args.warmup + args.steps) * k.use_count, t_us)  # the cold passes of the timed region
        same = (tr is None and na is None) or (tr is not None and na is not None and tr.knobs() == na.knobs())
        n_us = t_us if same else cold_launches(k, sets, na)
        e = by_name[k.name]
        per_kernel.append(dict(name=k.name, transfer_us=t_us, native_us=n_us, default_us_at_sweep=e["default_us"],
                               frac_of_native=min(n_us, t_us) / t_us, tflops=k.flops() / t_us / 1e6,
                               gbps=k.algorithmic_bytes() / t_us / 1e3, kernel=symbol_of(k, tr), tensor_sets=n_sets,
                               on_default_fallback=tr is None))
        del sets
        torch.cuda.empty_cache()
    fracs = [p["frac_of_native"] for p in per_kernel]

    # the dominant kernel symbol: the one with the largest share of a pass (use counts x cold durations)
    share = {}
    for p, k in zip(per_kernel, targets):
        g = share.setdefault(p["kernel"], dict(us=0.0, flops=0.0, bytes=0.0, launches=0))
        g["us"] += p["transfer_us"] * k.use_count
        g["flops"] += k.flops() * k.use_count
        g["bytes"] += k.algorithmic_bytes() * k.use_count
        g["launches"] += k.use_count
    pass_us = sum(g["us"] for g in share.values())

    def roofline_of(name, in_pass):
        led = ledger[name]
        peak = PEAK["mfma_bf16"] if led["dtype"] == wl.BF16 else PEAK["mfma_f32"]
        ai = in_pass["flops"] / in_pass["bytes"]
        if ai >= peak * 1e12 / (PEAK["hbm"] * 1e9):
            roof = dict(bound="mfma", achieved=in_pass["flops"] / in_pass["us"] / 1e6, peak=peak, unit="TFLOP/s")
        else:
            roof = dict(bound="hbm", achieved=in_pass["bytes"] / in_pass["us"] / 1e3, peak=PEAK["hbm"], unit="GB/s")
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof["share_of_pass"] = in_pass["us"] / pass_us
        roof["launches_per_pass"] = in_pass["launches"]
        # HBM bytes per launch measured with rocprofv3 counters (paper_2201_05587_amd/traffic.py), reported
        # only while the kernel sources are the ones the counters were taken on
        roof["traffic"] = traffic.lookup(args.workload, name)
        roof.update(kernel=name, avg_launch_us=in_pass["us"] / in_pass["launches"],
                    avg_launch_us_all_launches_of_this_process=led["us"] / led["launches"], launches=led["launches"],
                    layers=sorted(led["layers"]), arithmetic_intensity=ai,
                    timing="cold: every launch on tensors that have left the caches")
        return roof

    by_share = sorted(share.items(), key=lambda kv: -kv[1]["us"])
    roof = roofline_of(*by_share[0])
    ridge_peak = PEAK["mfma_bf16"] if ledger[by_share[0][0]]["dtype"] == wl.BF16 else PEAK["mfma_f32"]
    # the symbol with the largest share among those bound by memory, and among those bound by the matrix cores
    roof_by_bound = {}
    for name, in_pass in by_share:
        r = roofline_of(name, in_pass)
        roof_by_bound.setdefault(r["bound"], r)
    groups = {n: dict(g, layers=sorted(g["layers"]), avg_us=g["us"] / g["launches"]) for n, g in ledger.items()}
    # the matrix-core-bound layers (arithmetic intensity above the ridge) against the MFMA peak
    mfma_bound = [dict(name=p["name"], tflops=p["tflops"], frac_of_mfma_peak=p["tflops"] / ridge_peak)
                  for p, k in zip(per_kernel, targets)
                  if k.flops() / k.algorithmic_bytes() >= ridge_peak * 1e12 / (PEAK["hbm"] * 1e9)]

    sweep = {"swept_in_this_run": False, "pairs": tuned["transfer_pairs"], "wall_seconds": tuned["transfer_wall_seconds"],
             "invalid_pairs": tuned["transfer_invalid_pairs"], "native_wall_seconds": tuned["native_wall_seconds"],
             "pool_records": tuned["pool_records"]}
    if swept_here:
        sweep["swept_in_this_run"] = True
    elif not args.no_live_sweep and not args.kernels:
        sweep = live_sweeps(args, api, tune, targets, dks, tune.load_pool(pool_path), by_name)

    out = {
        "metric": "fused-op TFLOP/s of best transferred schedule; % of native-swept optimum",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if targets[0].shape.dtype == wl.BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {len(targets)} fused kernels, {sum(k.use_count for k in targets)} "
                               f"launches per pass, {pass_flops / 1e9:.1f} GFLOP and {pass_bytes / 1e6:.0f} MB of "
                               f"compulsory traffic per pass; tensors channels-last (NHWC activations, KRSC filters)",
                   "pool_records": tuned["pool_records"], "swept_in_this_run": sweep["swept_in_this_run"],
                   "kernels_on_default_fallback": sum(1 for t in transfer if t is None)},
        "cold": {"ms_per_step": ms_per_step, "tflops": value,
                 "what": "every launch of a pass on tensors of its own (the headline)"},
        "warm": {"ms_per_step": warm_ms, "tflops": pass_flops / warm_ms / 1e9,
                 "what": "each kernel's use_count launches repeated on one set of tensors"},
        "pct_of_native_optimum": {"mean": 100.0 * sum(fracs) / len(fracs), "min": 100.0 * min(fracs),
                                  "kernels_at_or_above_80pct": sum(f >= 0.8 for f in fracs), "kernels": len(fracs)},
        "mfma_bound_layers": mfma_bound,
        "sweep": sweep,
        "roofline": roof,
        "roofline_by_bound": roof_by_bound,
    }
    out["machine_rates"] = machine_rates(api)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_leg(wl, targets)
    report = os.path.join(ROOT, "gpurun_out", f"bench_{args.workload}_kernels.json")
    if os.path.isdir(os.path.dirname(report)):
        tune.save_json(report, dict(per_kernel=per_kernel, groups=groups))
    for p in per_kernel:
        log(f"{p['name']:34s} transfer {p['transfer_us']:9.2f} us  native {p['native_us']:9.2f}  "
            f"{p['tflops']:8.1f} TFLOP/s {p['gbps']:8.1f} GB/s  frac {p['frac_of_native']:.3f}  {p['kernel']}")
    for n, g in sorted(groups.items(), key=lambda kv: -kv[1]["us"]):
        log(f"[symbol] {n:60s} launches {g['launches']:6d}  avg {g['avg_us']:9.2f} us  total {g['us'] / 1e3:9.2f} ms")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
