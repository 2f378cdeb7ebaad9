"""The conv entry point that allocates nothing (split-K partials in the library's static array) against
the ordinary entry point with a caller's workspace: same kernels, so the outputs are equal bit for bit.
Two calls in a row on one GPU, the second on a smaller input, share the array."""
import pytest

from paper_2201_05587_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_both(api, harness, kernel, sched, seed):
    import torch
    dk = harness.device_kernel(kernel, seed)
    t = dk.tensors
    want = torch.full_like(t["y"], float("nan"))
    got = torch.full_like(t["y"], float("nan"))
    plan = api.tt_schedule_apply(sched, kernel.cls, kernel.shape)
    assert plan.status == api.TT_OK and plan.variant_id >= 0 and plan.eff_split_k > 1
    assert 0 < plan.workspace_bytes <= api.TT_STATIC_WORKSPACE_BYTES
    api.tt_conv2d_bias_relu(t["x"], t["w"], t["bias"], t.get("res"), kernel.shape, kernel.cls, sched, ws=dk.ws, y=want)
    rc = api.tt_conv2d_bias_relu_noalloc(t["x"], t["w"], t["bias"], t.get("res"), got, kernel.shape, kernel.cls, sched)
    torch.cuda.synchronize()
    assert rc == api.TT_OK, api.status_name(rc)
    assert bool(torch.isfinite(want).all()) and bool(torch.isfinite(got).all())
    assert torch.equal(got.view(torch.int32 if got.dtype == torch.float32 else torch.int16),
                       want.view(torch.int32 if want.dtype == torch.float32 else torch.int16))
    return got


def test_static_workspace_entry_point_matches_the_ordinary_one_on_two_calls_in_a_row():
    import torch
    from paper_2201_05587_amd import api, harness
    import parity
    E, F = wl.CLS_CONV2D_BIAS_RELU, wl.CLS_CONV2D_BIAS_ADD_RELU
    # first call: 3x3 conv on a 14 x 14 map, batch 4, bf16, reduction split four ways (3.2 MB of partials)
    big = wl.Kernel(E, wl.ConvShape(4, 256, 14, 14, 256, 3, 3, 1, 1, 1, 1, wl.BF16), 1, "noalloc_big")
    s_big = api.make_schedule(E, api.TT_SK_MFMA, 64, 64, 64, 32, 32, 32, 4, 0, 8, 8, 3)
    out_big = run_both(api, harness, big, s_big, 4242)
    # second call, smaller input, other class and data type: ragged tiles, residual, three splits of fp32
    small = wl.Kernel(F, wl.ConvShape(1, 40, 9, 9, 24, 3, 3, 1, 1, 1, 1, wl.F32), 1, "noalloc_small")
    s_small = api.make_schedule(F, api.TT_SK_MFMA, 32, 16, 32, 32, 16, 16, 3, 1, 4, 8, 2)
    out_small = run_both(api, harness, small, s_small, 4343)
    # and both against the oracle, to the bar of every other parity test
    for k, out, seed in ((big, out_big, 4242), (small, out_small, 4343)):
        inp = wl.make_inputs(k, seed)
        ref = parity.oracle_output(k, inp)
        got = harness.output_in_definition_order(k, out).float().cpu().numpy()
        parity.assert_close(got, ref, k.shape.dtype, k.name)


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    import torch
    from paper_2201_05587_amd import api, harness
    E = wl.CLS_CONV2D_BIAS_RELU
    # 32 x 28 x 28 x 256 outputs, two splits: 51 MB of partial sums
    k = wl.Kernel(E, wl.ConvShape(32, 64, 28, 28, 256, 3, 3, 1, 1, 1, 1, wl.BF16), 1, "noalloc_too_big")
    sched = api.make_schedule(E, api.TT_SK_MFMA, 64, 64, 64, 32, 32, 32, 2, 0, 8, 8, 2)
    plan = api.tt_schedule_apply(sched, k.cls, k.shape)
    assert plan.status == api.TT_OK and plan.workspace_bytes > api.TT_STATIC_WORKSPACE_BYTES
    dk = harness.device_kernel(k, 7, max_split=1)
    t = dk.tensors
    t["y"].fill_(float("nan"))
    rc = api.tt_conv2d_bias_relu_noalloc(t["x"], t["w"], t["bias"], None, t["y"], k.shape, k.cls, sched)
    torch.cuda.synchronize()
    assert rc == api.TT_ERR_WORKSPACE
    assert b"static workspace" in api.lib.tt_last_error()
    assert bool(torch.isnan(t["y"]).all())  # nothing was launched
    # without a split the same kernel needs no workspace and runs
    rc = api.tt_conv2d_bias_relu_noalloc(t["x"], t["w"], t["bias"], None, t["y"], k.shape, k.cls, None)
    torch.cuda.synchronize()
    assert rc == api.TT_OK and bool(torch.isfinite(t["y"]).all())
