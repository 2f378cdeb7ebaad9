"""Helpers of the GPU parity tests: run a kernel through the C-ABI, compute the oracle, compare."""
import numpy as np

from oracle import ops as O
from paper_2201_05587_amd import api, harness
from paper_2201_05587_amd import workloads as wl

TOL = {wl.F32: 1e-4, wl.BF16: 2e-2}


def oracle_output(kernel: wl.Kernel, inp: dict) -> np.ndarray:
    s = kernel.shape
    act = wl.CLASS_ACT[kernel.cls]
    if kernel.cls == wl.CLS_DWCONV_BIAS_RELU6:
        return O.dwconv(inp["x"], inp["w"], inp["bias"], (s.stride_h, s.stride_w), (s.pad_h, s.pad_w), act)
    if kernel.is_conv():
        return O.conv2d(inp["x"], inp["w"], inp["bias"], inp.get("res"), (s.stride_h, s.stride_w),
                        (s.pad_h, s.pad_w), act)
    if kernel.cls == wl.CLS_BATCH_MATMUL:
        return O.batch_matmul(inp["a"], inp["b"], bool(s.trans_b))
    return O.dense(inp["x"], inp["w"], inp["bias"], act)


def assert_close(got: np.ndarray, ref: np.ndarray, dtype: int, what=""):
    """|g - r| <= tol * (|r| + rms(r)) for every element, and max|g - r| <= tol * max|r|."""
    tol = TOL[dtype]
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(got - ref)
    bound = tol * (np.abs(ref) + rms)
    bad = err > bound
    assert not bad.any(), (what, int(bad.sum()), float(err.max()), float(err[bad].max()), rms,
                           np.argwhere(bad)[:4].tolist())
    assert err.max() <= tol * max(np.abs(ref).max(), 1e-30), (what, float(err.max()))


def run_gpu(kernel: wl.Kernel, dk: api.DeviceKernel, sched=None) -> np.ndarray:
    """Run once and return the output in the definition's index order ([n,k,Ho,Wo] for conv)."""
    import torch
    dk.output().fill_(float("nan"))
    rc = dk.run(sched)
    torch.cuda.synchronize()
    assert rc == api.TT_OK, (api.status_name(rc), sched)
    return harness.output_in_definition_order(kernel, dk.output()).float().cpu().numpy()


def check_kernel(kernel: wl.Kernel, scheds, seed=1234, ref=None):
    """Run `kernel` under each record in `scheds` (None = default) and compare with the oracle."""
    inp = wl.make_inputs(kernel, seed)
    if ref is None:
        ref = oracle_output(kernel, inp)
    dk = harness.device_kernel(kernel, seed, inp)
    outs = []
    for s in scheds:
        if s is not None:
            # records the integer oracle rejects for this shape must be rejected by the library, unlaunched
            from oracle import schedule as S
            from test_oracle_schedule import oshape
            want = S.apply({f: getattr(s, f) for f in S.RECORD_FIELDS}, kernel.cls, oshape(kernel))["status"]
            if want != S.OK:
                assert dk.run(s) == want, (kernel.name, s)
                outs.append(None)
                continue
        if s is not None:
            plan = api.tt_schedule_apply(s, kernel.cls, kernel.shape)
            if plan.status != api.TT_OK:
                # refused for a reason of the library's own kernels (LDS size, K step): nothing launched
                assert plan.status == api.TT_ERR_INVALID_SCHEDULE and plan.reason in (6, 7), (kernel.name, s)
                assert dk.run(s) == api.TT_ERR_INVALID_SCHEDULE
                outs.append(None)
                continue
            if plan.variant_id < 0:
                # a valid plan no compiled kernel implements: refused, nothing launched
                assert dk.run(s) == api.TT_ERR_UNSUPPORTED, (kernel.name, s)
                outs.append(None)
                continue
        got = run_gpu(kernel, dk, s)
        assert_close(got, ref, kernel.shape.dtype, f"{kernel.name} {s}")
        outs.append(got)
    return ref, outs
