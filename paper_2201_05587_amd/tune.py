"""Sweeps over schedule records: native (exhaustive) tuning of a kernel, donor pools, pool files.

All timing and selection run inside the library (``tt_transfer_sweep``); this module only prepares
the arguments, keeps the records with their provenance and reads / writes the pool file, the
reusable artefact of transfer-tuning (the paper's "auto-schedules of pre-tuned models", Section 4.3).
"""
from __future__ import annotations

import json
import time
from typing import Dict, List, Optional, Sequence

from . import api, harness
from . import workloads as wl

POOL_MAGIC = "# tt-pool v1: cls sketch tile_m tile_n tile_k wave_m wave_n mfma split_k order vec unroll stages | donor shape | donor_us | donor name"

# cheap protocol for walking a large space, full protocol (paper Section 5.1: median of 10) for the finalists
EXPLORE = dict(warmup=1, samples=3, min_sample_us=60, max_launches=16)
FULL = dict(warmup=3, samples=10, min_sample_us=200, max_launches=64)


def shape_ints(shape) -> List[int]:
    cs = api.to_c_shape(shape)
    vals = [getattr(cs, f) for f, _ in cs._fields_]
    return vals + [0] * (12 - len(vals))


def native_sweep(dk: api.DeviceKernel, level: int = 1, finalists: int = 4):
    """Exhaustive sweep of the class's schedule space on the kernel's own shape (runs in the library).

    Returns (best_record, best_us, default_us, n_valid, n_records); the record is None when nothing
    beats the default schedule.
    """
    best, best_us, default_us, n_valid, n_rec = api.tt_native_sweep(dk, level, finalists, api.make_opts(**EXPLORE),
                                                                    api.make_opts(**FULL))
    default = api.tt_schedule_default(dk.cls, dk.cshape)
    return (None if best.knobs() == default.knobs() else best), best_us, default_us, n_valid, n_rec


def fastest_distinct_tiles(dk: api.DeviceKernel, level: int, count: int, tiles=(32, 64, 128)):
    """The `count` fastest records of the class's space on this kernel whose workgroup tiles come from
    `tiles` and differ pairwise in (tile_m, tile_n, tile_k): a small donor pool from one tuned kernel."""
    space = [r for r in api.tt_schedule_space(dk.cls, dk.cshape.dtype, level)
             if r.sketch == api.TT_SK_MFMA and r.tile_m in tiles and r.tile_n in tiles and r.tile_k in tiles]
    _, table, _, _ = api.tt_transfer_sweep([dk], space, api.make_opts(**EXPLORE))
    ranked = sorted((t, i) for i, t in enumerate(table[0]) if t >= 0)
    top, seen = [], set()
    for _, i in ranked:
        key = (space[i].tile_m, space[i].tile_n, space[i].tile_k)
        if key not in seen:
            seen.add(key)
            top.append(space[i])
        if len(top) == 3 * count:
            break
    _, table, _, _ = api.tt_transfer_sweep([dk], top, api.make_opts(**FULL))
    ranked = sorted((t, i) for i, t in enumerate(table[0]) if t >= 0)[:count]
    return [(top[i].copy(), t) for t, i in ranked]


def tune_donors(kernels: Sequence[wl.Kernel], seed_cfg: int, level: int = 1, log=None,
                records_per_donor: int = 1, checkpoint: Optional[str] = None,
                resume: Optional[str] = None, cold_mb: float = 0.0, cold_min_mb: float = 0.0) -> List[api.tt_schedule]:
    """Native-tune every donor kernel; each contributes its optimum as one pool record (or, with
    records_per_donor > 1, its fastest records of pairwise distinct workgroup tiles).

    With `checkpoint` the pool so far is written to that file after every donor; `resume` names such a
    file of an earlier run, whose donors are not tuned again (a long tuning job may be cut short).
    cold_mb, cold_min_mb: megabytes of tensor sets every pair's launches rotate through (0: one set, cache-warm
    timing), for donors whose tensors take at least cold_min_mb.
    """
    import os
    import torch
    pool: List[api.tt_schedule] = []
    done = 0
    if resume and os.path.exists(resume) and records_per_donor == 1:
        pool = load_pool(resume)
        done = len(pool)
        if log:
            log(f"[pool] continuing after {done} donors found in {resume}")
    for i, k in enumerate(kernels):
        if i < done:
            continue
        if checkpoint and records_per_donor == 1 and pool:
            save_pool(checkpoint, pool, [kk.name for kk in kernels[:len(pool)]])
        dk = harness.device_kernel(k, wl.seed_for(seed_cfg, i), max_split=8, cold_mb=cold_mb, cold_min_mb=cold_min_mb)
        t0 = time.time()
        if records_per_donor > 1:
            for rec, us in fastest_distinct_tiles(dk, level, records_per_donor):
                rec.id = len(pool)
                for j, v in enumerate(shape_ints(k.shape)):
                    rec.donor_shape[j] = v
                rec.donor_us = us
                pool.append(rec)
                if log:
                    log(f"donor {i:3d} {k.name:34s} {us:9.2f} us  {rec}")
            del dk
            torch.cuda.empty_cache()
            continue
        best, best_us, default_us, n_valid, n_rec = native_sweep(dk, level)
        if best is None:
            best = api.tt_schedule_default(k.cls, k.shape)
        best.id = len(pool)
        for j, v in enumerate(shape_ints(k.shape)):
            best.donor_shape[j] = v
        best.donor_us = best_us
        pool.append(best)
        if log:
            log(f"donor {i:3d} {k.name:34s} best {best_us:9.2f} us (default {default_us:9.2f}) "
                f"{n_valid}/{n_rec} valid, {time.time() - t0:.1f}s  {best}")
        del dk
        torch.cuda.empty_cache()
    return pool


def save_pool(path: str, pool: Sequence[api.tt_schedule], names: Optional[Sequence[str]] = None) -> None:
    with open(path, "w") as f:
        f.write(POOL_MAGIC + "\n")
        for i, r in enumerate(pool):
            knobs = " ".join(str(getattr(r, k)) for k in api.tt_schedule.KNOBS)
            shape = " ".join(str(v) for v in r.donor_shape)
            f.write(f"{knobs} | {shape} | {r.donor_us:.3f} | {names[i] if names else ''}\n")


def load_pool(path: str) -> List[api.tt_schedule]:
    pool = []
    with open(path) as f:
        head = f.readline()
        if not head.startswith("# tt-pool v1"):
            raise ValueError(f"{path}: not a tt-pool v1 file")
        for ln in f:
            ln = ln.strip()
            if not ln or ln.startswith("#"):
                continue
            knobs, shape, us, _ = [p.strip() for p in ln.split("|")]
            vals = [int(v) for v in knobs.split()]
            r = api.make_schedule(*vals, id=len(pool))
            for j, v in enumerate(int(x) for x in shape.split()):
                r.donor_shape[j] = v
            r.donor_us = float(us)
            pool.append(r)
    return pool


# ---- which pool to transfer from (paper Section 4.4.2, Eq. 1) -------------------------------------------
def choose_donor_pool(targets: Sequence[wl.Kernel], default_us: Sequence[float], pools: Dict[str, Sequence[api.tt_schedule]]):
    """Rank candidate pools for a target network: (best name, {name: score}).

    P_c is the share of class c in the target's time under the default schedules (each kernel's time
    counted as often as the network uses it); |W_Tc| is the number of records of class c in a pool.
    The arithmetic runs in the library (``tt_select_donor``).
    """
    cost = [0.0] * api.TT_NUM_CLASSES
    for k, us in zip(targets, default_us):
        cost[k.cls] += float(us) * k.use_count
    names = list(pools)
    counts = [[sum(1 for r in pools[n] if r.cls == c) for c in range(api.TT_NUM_CLASSES)] for n in names]
    best, scores = api.tt_select_donor(cost, counts)
    return (names[best] if best >= 0 else None), dict(zip(names, scores))


# ---- workloads: target kernels and the donor kernels whose native optima form the pool -------------
def workload(name: str):
    """(cfg index, target kernels, donor kernels) of a named configuration."""
    if name == "cfg1":
        # one donor kernel; its pool holds its 4 fastest records of distinct tiles from {32, 64, 128}^3
        return 1, [wl.cfg1_target()], [wl.cfg1_donor()]
    if name == "cfg2":
        return 2, wl.resnet18_kernels(1, wl.F32), wl.resnet50_kernels(1, wl.F32)
    if name == "cfg3":
        donors = wl.bert_kernels(seq=256) + wl.bert_kernels(seq=128, hidden=512, heads=4, ffn=2048) + \
            wl.bert_kernels(seq=256, hidden=512, heads=4, ffn=512)
        return 3, wl.bert_kernels(seq=128), donors
    if name == "cfg4":
        return 4, wl.mobilenetv2_kernels(16, wl.F32), wl.mobilenetv2_kernels(1, wl.F32) + \
            [k for k in wl.resnet50_kernels(1, wl.F32) if k.is_conv()][:8]
    if name == "cfg5":
        targets = wl.resnet50_kernels(32, wl.BF16, with_dense=False)
        exclude = {(k.cls, k.shape) for k in targets}
        donors = []
        for i in range(10):
            donors += wl.synthetic_network(i, 32, wl.BF16, 30, exclude)
        return 5, targets, donors
    # sequence-length transfer (paper Section 5.4): schedules tuned at one length applied at the other
    if name == "seq128_from_256":
        return 3, wl.bert_kernels(seq=128), wl.bert_kernels(seq=256)
    if name == "seq256_from_128":
        return 3, wl.bert_kernels(seq=256), wl.bert_kernels(seq=128)
    raise ValueError(f"unknown workload {name}")


def save_json(path: str, obj) -> None:
    with open(path, "w") as f:
        json.dump(obj, f, indent=1)
        f.write("\n")
