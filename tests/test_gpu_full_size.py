"""Parity at the full sizes of the evaluation configurations, in the launch configuration bench.py times.

Every kernel of every configuration runs under the default record, under the record the stored
transfer sweep chose and under the native-swept one, i.e. the records the timed pass launches, and
its whole output tensor is compared with the oracle element by element.  A stored record that no
longer applies to its kernel, or that no compiled kernel implements, is a failure, not a skip.  The
ResNet50-shaped batch-32 kernels are additionally checked on sampled outputs the point-wise oracle
computes one by one (a fast pre-check that names the failing coordinates).
"""
import json
import os

import numpy as np
import pytest

from oracle import ops as O
from paper_2201_05587_amd import api, harness, tune
from paper_2201_05587_amd import workloads as wl
from parity import TOL, assert_close, check_kernel, run_gpu

pytestmark = pytest.mark.gpu

TUNED_DIR = os.path.join(os.path.dirname(os.path.abspath(api.__file__)), "tuned")
KNOBS = ("cls", "sketch", "tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "mfma", "split_k", "order", "vec",
         "unroll", "stages")


def stored_records(workload: str):
    """name -> list of records (transfer choice, native choice) of the committed sweep outcome."""
    path = os.path.join(TUNED_DIR, f"{workload}.json")
    assert os.path.exists(path), f"no stored sweep outcome for {workload}"
    with open(path) as f:
        tuned = json.load(f)
    out = {}
    for e in tuned["kernels"]:
        recs = []
        for key in ("transfer", "native"):
            kn = e.get(key)
            if kn:
                recs.append(api.make_schedule(**{f: kn[f] for f in KNOBS}))
        out[e["name"]] = recs
    return out


def records_to_check(workload: str, kernel: wl.Kernel):
    """[default] + the stored records of the kernel, each of which must be a plan a kernel implements."""
    stored = stored_records(workload)
    assert kernel.name in stored, (workload, kernel.name, "kernel missing from the stored sweep outcome")
    for rec in stored[kernel.name]:
        plan = api.tt_schedule_apply(rec, kernel.cls, kernel.shape)
        assert plan.status == api.TT_OK, (kernel.name, rec, api.status_name(plan.status), plan.reason)
        assert plan.variant_id >= 0, (kernel.name, rec, "no compiled kernel implements this stored record")
    return [None] + stored[kernel.name]


def sample_coords(kernel: wl.Kernel, count: int, seed: int) -> np.ndarray:
    """Uniform output coordinates plus all four corners, edge rows and edge columns for some (n, k)."""
    s = kernel.shape
    g = np.random.default_rng(seed)
    pts = np.stack([g.integers(0, s.n, count), g.integers(0, s.k, count), g.integers(0, s.ho, count),
                    g.integers(0, s.wo, count)], axis=1)
    edge = []
    for n in (0, s.n - 1):
        for k in (0, s.k // 2, s.k - 1):
            for p in (0, 1, s.ho // 2, s.ho - 1):
                for q in range(s.wo):
                    edge.append((n, k, p, q))
            for q in (0, s.wo - 1):
                for p in range(s.ho):
                    edge.append((n, k, p, q))
    # the last rows of the flattened pixel axis and the last output channels: ragged tile tails
    for k in range(max(0, s.k - 8), s.k):
        for q in range(s.wo):
            edge.append((s.n - 1, k, s.ho - 1, q))
    return np.concatenate([pts, np.array(edge, dtype=np.int64)], axis=0).astype(np.int32)


def cfg5_cases():
    _, targets, _ = tune.workload("cfg5")
    return [pytest.param(i, id=k.name) for i, k in enumerate(targets)]


@pytest.mark.parametrize("index", cfg5_cases())
def test_cfg5_full_size_sampled(index):
    import torch
    cfg, targets, _ = tune.workload("cfg5")
    kernel = targets[index]
    s = kernel.shape
    seed = wl.seed_for(cfg, index)
    inp = wl.make_inputs(kernel, seed)
    coords = sample_coords(kernel, 4000, seed)
    act = wl.CLASS_ACT[kernel.cls]
    ref = O.conv2d_points(inp["x"], inp["w"], coords, inp["bias"], inp.get("res"), (s.stride_h, s.stride_w),
                          (s.pad_h, s.pad_w), act)
    dk = harness.device_kernel(kernel, seed, inp)
    scheds = records_to_check("cfg5", kernel)
    ix = tuple(torch.from_numpy(coords[:, j].astype(np.int64)).cuda() for j in range(4))
    for rec in scheds:
        dk.output().fill_(float("nan"))
        rc = dk.run(rec)
        torch.cuda.synchronize()
        assert rc == api.TT_OK, (kernel.name, rec, api.status_name(rc))
        y = harness.output_in_definition_order(kernel, dk.output())
        assert bool(torch.isfinite(y).all()), (kernel.name, rec, "unwritten or non-finite outputs")
        if act == wl.ACT_RELU:
            assert float(y.min()) >= 0.0
        got = y[ix].float().cpu().numpy()
        # same bound as the whole-tensor comparison; the rms of the sample stands in for the tensor's
        assert_close(got, ref, s.dtype, f"{kernel.name} {rec}")


def whole_config(name):
    cfg, targets, _ = tune.workload(name)
    return cfg, targets


def cases_of(name):
    _, targets = whole_config(name)
    return [pytest.param(i, id=k.name) for i, k in enumerate(targets)]


def run_whole(name, index):
    cfg, targets = whole_config(name)
    kernel = targets[index]
    _, outs = check_kernel(kernel, records_to_check(name, kernel), seed=wl.seed_for(cfg, index))
    assert all(o is not None for o in outs), (name, kernel.name, "a stored record was refused")


@pytest.mark.parametrize("index", cfg5_cases())
def test_cfg5_resnet50_b32_bf16_whole(index):
    """The batch-32 kernels whole: the oracle computes all 24 layers in seconds on the host cores."""
    run_whole("cfg5", index)


@pytest.mark.parametrize("index", cases_of("cfg1"))
def test_cfg1_conv_fp32_whole(index):
    """The single convolution of the smallest configuration under the records its four-record pool gave it."""
    run_whole("cfg1", index)


@pytest.mark.parametrize("index", cases_of("cfg2"))
def test_cfg2_resnet18_fp32_whole(index):
    run_whole("cfg2", index)


@pytest.mark.parametrize("index", cases_of("cfg3"))
def test_cfg3_bert_bf16_whole(index):
    run_whole("cfg3", index)


@pytest.mark.parametrize("index", cases_of("cfg4"))
def test_cfg4_mobilenetv2_fp32_whole(index):
    run_whole("cfg4", index)


@pytest.mark.parametrize("index", cases_of("seq128_from_256"))
def test_seq128_bert_bf16_whole(index):
    """Targets at sequence length 128 under the records transferred from length 256 (Section 5.4)."""
    run_whole("seq128_from_256", index)


@pytest.mark.parametrize("index", cases_of("seq256_from_128"))
def test_seq256_bert_bf16_whole(index):
    """Targets at sequence length 256 under the records transferred from length 128 (Section 5.4)."""
    run_whole("seq256_from_128", index)
