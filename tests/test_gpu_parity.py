"""GPU parity: every operator class through the C-ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

from oracle import schedule as S
from paper_2201_05587_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_2201_05587_amd import api as _api
    return _api


@pytest.fixture(scope="module")
def P():
    import parity
    return parity


def mfma(api, cls, tm, tn, tk, wm, wn, mf, split_k=1, order=0, vec=8, unroll=8, stages=2):
    return api.make_schedule(cls, api.TT_SK_MFMA, tm, tn, tk, wm, wn, mf, split_k, order, vec, unroll, stages)


def conv_kernel(cls, n, c, hw, k, f, stride, dtype=wl.F32, pad=None):
    pad = f // 2 if pad is None else pad
    return wl.Kernel(cls, wl.ConvShape(n, c, hw, hw, k, f, f, stride, stride, pad, pad, dtype), 1,
                     f"conv{f}x{f}_{c}_{k}_{hw}_s{stride}")


# ---- index map ------------------------------------------------------------------------------------
def test_device_index_map_matches_oracle_bit_for_bit(api):
    from test_host_schedule import to_c_record
    from test_oracle_schedule import oshape
    cases = [(wl.cfg1_target(), S.record(1, S.SK_MFMA, 32, 32, 32, 16, 16, 16, 4, o)) for o in range(6)]
    cases += [(wl.resnet18_kernels()[13], S.record(1, S.SK_MFMA, 32, 64, 32, 32, 32, 32, 7, 5))]
    cases += [(wl.bert_kernels()[5], S.record(7, S.SK_MFMA, 64, 64, 32, 32, 32, 16, 2, 2))]
    cases += [(wl.mobilenetv2_kernels(2)[3], S.record(8, S.SK_DWCONV, 4, 16, 4, 1, 1, 0, 1, 4, 1, 1, 1))]
    cases += [(wl.resnet50_kernels(32, wl.BF16, False)[0], S.record(1, S.SK_MFMA, 128, 64, 32, 64, 32, 32, 1, 5))]
    for k, rec in cases:
        oplan = S.apply(rec, k.cls, oshape(k))
        assert oplan["status"] == S.OK
        cplan = api.tt_schedule_apply(to_c_record(rec), k.cls, k.shape)
        dev = api.tt_debug_tile_map(cplan)
        want = np.array([S.plan_tile(oplan, wg) for wg in range(oplan["grid"])], dtype=np.int32)
        np.testing.assert_array_equal(dev, want)


# ---- conv2d classes, fp32 -------------------------------------------------------------------------
def test_cfg1_conv_under_default_and_donor_tiles(api, P):
    k = wl.cfg1_target()
    E = k.cls
    scheds = [None,
              mfma(api, E, 32, 32, 16, 16, 16, 16), mfma(api, E, 64, 64, 32, 32, 32, 32),
              mfma(api, E, 64, 32, 32, 32, 32, 16), mfma(api, E, 128, 64, 32, 64, 32, 32),
              mfma(api, E, 256, 64, 16, 64, 64, 32, order=1), mfma(api, E, 32, 64, 32, 32, 32, 32, stages=1, unroll=1),
              mfma(api, E, 64, 64, 16, 32, 32, 16, split_k=4, order=3), mfma(api, E, 16, 16, 32, 16, 16, 16, split_k=3),
              api.make_schedule(E, api.TT_SK_DIRECT, 1, 1, 1, 1, 1, 0, 1, 0, 1, 1, 1)]
    ref, outs = P.check_kernel(k, scheds)
    assert ref.min() >= 0.0
    # same (tile_k, split_k, block) => same summation order => identical bits, whatever the tile shape
    a = P.run_gpu(k, __import__("paper_2201_05587_amd.harness", fromlist=["x"]).device_kernel(k, 1234),
                  mfma(api, E, 64, 64, 32, 32, 32, 32))
    np.testing.assert_array_equal(a, outs[2])


@pytest.mark.parametrize("case", [
    ("stem7x7", wl.CLS_CONV2D_BIAS_RELU, (1, 3, 224, 64, 7, 2)),
    ("proj1x1s2", wl.CLS_CONV2D_ADD, (1, 64, 56, 128, 1, 2)),
    ("res3x3", wl.CLS_CONV2D_BIAS_ADD_RELU, (1, 128, 28, 128, 3, 1)),
    ("s2_3x3", wl.CLS_CONV2D_BIAS_RELU, (1, 128, 28, 256, 3, 2)),
    ("map7x7", wl.CLS_CONV2D_BIAS_ADD_RELU, (1, 512, 7, 512, 3, 1)),
    ("pw_relu6", wl.CLS_CONV2D_BIAS_RELU6, (2, 24, 56, 144, 1, 1)),
    ("pw_small_n", wl.CLS_CONV2D_ADD, (1, 96, 112, 24, 1, 1)),
    ("batch3_5x5", wl.CLS_CONV2D_BIAS_RELU, (3, 20, 19, 40, 5, 1)),
])
def test_conv_classes_and_shapes_fp32(api, P, case):
    name, cls, (n, c, hw, kk, f, st) = case
    k = conv_kernel(cls, n, c, hw, kk, f, st)
    scheds = [None, mfma(api, cls, 32, 32, 16, 16, 16, 16, order=1), mfma(api, cls, 16, 16, 16, 16, 16, 16, split_k=2),
              mfma(api, cls, 32, 16, 32, 32, 16, 16, order=5, stages=1)]
    if k.gemm_extents()[1] >= 64 and k.gemm_extents()[2] >= 64:
        scheds.append(mfma(api, cls, 64, 64, 32, 32, 32, 32, split_k=2, order=2))
    P.check_kernel(k, scheds)


def test_conv_bf16(api, P):
    for cls, dims in ((wl.CLS_CONV2D_BIAS_RELU, (2, 64, 28, 128, 3, 1)), (wl.CLS_CONV2D_BIAS_ADD_RELU, (2, 128, 14, 64, 1, 1)),
                      (wl.CLS_CONV2D_ADD, (2, 64, 28, 96, 1, 2)), (wl.CLS_CONV2D_BIAS_RELU, (1, 3, 64, 32, 7, 2))):
        k = conv_kernel(cls, *dims, dtype=wl.BF16)
        scheds = [None, mfma(api, cls, 32, 32, 32, 16, 16, 16), mfma(api, cls, 64, 64, 64, 32, 32, 32, split_k=2),
                  mfma(api, cls, 64, 32, 32, 32, 32, 32, order=4, stages=1, unroll=1)]
        P.check_kernel(k, scheds)


@pytest.mark.parametrize("dt", [wl.F32, wl.BF16])
@pytest.mark.parametrize("dims", [
    (2, 16, 56, 32, 3, 1),    # 16 channels: whole 16-byte items in both data types
    (3, 24, 14, 48, 3, 1),    # 24 channels, small odd-sized maps
    (2, 8, 16, 32, 5, 1),     # 5x5, pad 2: runs of 40 elements, two padded columns either side
    (1, 4, 24, 16, 7, 1),     # 7x7, pad 3, 4 channels: whole items in fp32, partly real items in bf16
    (2, 32, 12, 32, 3, 1),    # slices of 32 and 64 that end exactly on a pixel
    (5, 40, 7, 64, 3, 1),     # 40 channels: slices straddle pixels and filter rows; 7 x 7 maps
    (2, 48, 20, 96, 1, 1),    # unit-stride 1x1: the dense family
    (3, 36, 9, 64, 1, 1),     # 1x1 with 36 channels: whole fp32 items (dense family), partly real bf16 items (gather)
])
def test_conv_vector_gather_modes(api, P, dims, dt):
    n, c, hw, kk, f, st = dims
    cls = wl.CLS_CONV2D_BIAS_RELU
    k = conv_kernel(cls, n, c, hw, kk, f, st, dtype=dt)
    tk = 16 if dt == wl.F32 else 32
    scheds = [None, mfma(api, cls, 32, 32, tk, 16, 16, 16), mfma(api, cls, 64, 32, tk * 2, 32, 32, 32, split_k=2, stages=1),
              mfma(api, cls, 128, 32, tk, 32, 32, 32, order=1), mfma(api, cls, 16, 16, tk, 16, 16, 16, vec=2),
              mfma(api, cls, 256, 32, tk, 64, 32, 16, vec=1)]
    P.check_kernel(k, scheds, seed=77)


def test_conv_padding_wider_than_filter_centre(api, P):
    # pad larger than (filter - 1) / 2 makes the output wider than the input: whole filter columns fall outside
    for dt in (wl.F32, wl.BF16):
        k = conv_kernel(wl.CLS_CONV2D_ADD, 2, 8, 6, 16, 3, 1, dtype=dt, pad=2)   # 6x6 -> 8x8
        assert k.shape.wo == 8
        tk = 16 if dt == wl.F32 else 32
        P.check_kernel(k, [None, mfma(api, k.cls, 32, 16, tk, 16, 16, 16), mfma(api, k.cls, 64, 16, tk, 16, 16, 16)])


# ---- asynchronous ring pipeline (3 or 4 stages) ----------------------------------------------------------
@pytest.mark.parametrize("dt", [wl.F32, wl.BF16])
def test_async_ring_conv(api, P, dt):
    cls = wl.CLS_CONV2D_BIAS_ADD_RELU
    tk = 16 if dt == wl.F32 else 32
    for dims in ((2, 64, 28, 128, 3, 1),      # 3x3 with padding, K = 576: many slices
                 (3, 32, 15, 96, 3, 2),       # odd map, stride 2, ragged M and N tiles
                 (2, 16, 12, 64, 5, 1),       # 5x5: runs of 80 elements, slices straddle filter rows
                 (2, 64, 14, 64, 1, 1),       # unit-stride 1x1: dense family, K = 64 (fewer slices than stages)
                 (2, 128, 14, 64, 1, 2)):     # strided 1x1: gathered
        k = conv_kernel(cls, *dims, dtype=dt)
        scheds = [mfma(api, cls, 64, 64, tk, 32, 32, 16, stages=3), mfma(api, cls, 64, 64, tk * 2, 32, 32, 32, stages=4),
                  mfma(api, cls, 128, 64, tk * 2, 64, 32, 32, stages=3, split_k=2, order=4),
                  mfma(api, cls, 32, 32, tk, 16, 16, 16, stages=4, unroll=1),
                  mfma(api, cls, 64, 64, tk * 2, 32, 32, 32, stages=4, vec=2)]   # reformulated to two stages
        on_ring = 0
        for s_ in scheds:
            plan = api.tt_schedule_apply(s_, k.cls, k.shape)
            if plan.status == api.TT_OK and plan.stages >= 3:
                assert api.variant_name(plan).startswith("tt::contract_async_kernel")
                on_ring += 1
        assert on_ring >= 2, k.name   # the 32 x 32 tile (too few items per thread) and vec = 2 fall back to two stages
        P.check_kernel(k, scheds, seed=31)


def test_async_ring_dense_and_batch_matmul(api, P):
    for dt in (wl.F32, wl.BF16):
        tk = 16 if dt == wl.F32 else 32
        k = wl.Kernel(wl.CLS_DENSE_BIAS_GELU, wl.GemmShape(1, 200, 264, 328, 1, dt), 1, f"dense_async_{dt}")
        P.check_kernel(k, [mfma(api, k.cls, 64, 64, tk * 2, 32, 32, 32, stages=3), mfma(api, k.cls, 128, 128, tk, 64, 64, 32, stages=4),
                           mfma(api, k.cls, 32, 32, tk, 16, 16, 16, stages=3, split_k=3)])
        b = wl.Kernel(wl.CLS_BATCH_MATMUL, wl.GemmShape(5, 128, 72, 96, 1, dt), 1, f"bmm_async_{dt}")
        P.check_kernel(b, [mfma(api, b.cls, 64, 64, tk, 32, 32, 32, stages=4), mfma(api, b.cls, 32, 32, tk * 2, 16, 16, 16, stages=3, order=4)])
        # K not a multiple of the 16-byte items: the ring does not apply and the record runs with two stages
        odd = wl.Kernel(wl.CLS_DENSE_BIAS_RELU, wl.GemmShape(1, 70, 90, 150, 1, dt), 1, f"dense_oddk_{dt}")
        rec = mfma(api, odd.cls, 32, 32, tk, 16, 16, 16, stages=3)
        assert api.tt_schedule_apply(rec, odd.cls, odd.shape).stages == 2
        P.check_kernel(odd, [rec])


def test_async_ring_with_fewer_slices_than_stages_and_at_the_loop_boundaries(api, P):
    """1..6 slices under 3 and 4 stages: prologue only, drain only, and one or more steady-state iterations."""
    for dt in (wl.F32, wl.BF16):
        tk = 16 if dt == wl.F32 else 32
        for slices in (1, 2, 3, 4, 5, 6):
            k = wl.Kernel(wl.CLS_DENSE_BIAS_RELU, wl.GemmShape(1, 96, 80, tk * slices, 1, dt), 1, f"dense_{slices}slices_{dt}")
            scheds = [mfma(api, k.cls, 64, 64, tk, 32, 32, 16, stages=3), mfma(api, k.cls, 64, 64, tk, 32, 32, 16, stages=4)]
            if slices >= 3:
                scheds.append(mfma(api, k.cls, 64, 64, tk, 32, 32, 16, stages=4, split_k=2))   # uneven halves
            for s_ in scheds:
                assert api.variant_name(api.tt_schedule_apply(s_, k.cls, k.shape)).startswith("tt::contract_async_kernel")
            P.check_kernel(k, scheds, seed=slices)
            c = conv_kernel(wl.CLS_CONV2D_BIAS_RELU, 1, tk * slices, 6, 32, 1, 2, dtype=dt)   # strided 1x1: gathered, K = C
            if c.shape.c % (8 if dt == wl.BF16 else 4) == 0:
                P.check_kernel(c, [mfma(api, c.cls, 32, 32, tk, 16, 16, 16, stages=4), mfma(api, c.cls, 64, 32, tk, 32, 16, 16, stages=3)],
                               seed=slices + 10)


# ---- dense / batch matmul -------------------------------------------------------------------------
def test_dense_classes(api, P):
    for cls in (wl.CLS_DENSE_ADD, wl.CLS_DENSE_BIAS_RELU, wl.CLS_DENSE_BIAS_GELU):
        for dt in (wl.F32, wl.BF16):
            k = wl.Kernel(cls, wl.GemmShape(1, 200, 264, 328, 1, dt), 1, f"dense_{cls}_{dt}")
            tk = 16 if dt == wl.F32 else 32
            scheds = [None, mfma(api, cls, 64, 64, tk * 2, 32, 32, 32), mfma(api, cls, 32, 32, tk, 16, 16, 16, split_k=3),
                      mfma(api, cls, 128, 128, tk, 64, 64, 32, order=1),
                      api.make_schedule(cls, api.TT_SK_DIRECT, 1, 1, 1, 1, 1, 0, 1, 0, 1, 1, 1)]
            P.check_kernel(k, scheds)


def test_dense_odd_k_uses_narrow_loads(api, P):
    for dt, kdim in ((wl.F32, 147), (wl.BF16, 150), (wl.BF16, 148), (wl.F32, 150)):
        k = wl.Kernel(wl.CLS_DENSE_BIAS_RELU, wl.GemmShape(1, 70, 90, kdim, 1, dt), 1, f"dense_k{kdim}")
        tk = 16 if dt == wl.F32 else 32
        P.check_kernel(k, [None, mfma(api, k.cls, 32, 32, tk, 16, 16, 16, vec=8), mfma(api, k.cls, 32, 32, tk, 16, 16, 16, vec=2)])


def test_output_rows_of_every_vector_width(api, P):
    """N a multiple of 8, of 4, of 2 and odd: whole-vector epilogue, and the element loop, with bias,
    residual, every activation class and split reductions (raw sums to the workspace)."""
    for dt in (wl.F32, wl.BF16):
        tk = 16 if dt == wl.F32 else 32
        for n in (96, 92, 90, 91):
            for cls in (wl.CLS_DENSE_ADD, wl.CLS_DENSE_BIAS_GELU):
                k = wl.Kernel(cls, wl.GemmShape(1, 70, n, 8 * tk, 1, dt), 1, f"dense_n{n}_{cls}_{dt}")
                P.check_kernel(k, [mfma(api, cls, 32, 32, tk, 16, 16, 16), mfma(api, cls, 64, 64, tk, 32, 32, 32, split_k=2),
                                   mfma(api, cls, 64, 64, tk * 2, 32, 32, 16, stages=3)], seed=n)
            c = conv_kernel(wl.CLS_CONV2D_BIAS_ADD_RELU, 2, 16, 9, n, 3, 1, dtype=dt)
            P.check_kernel(c, [mfma(api, c.cls, 64, 32, tk, 32, 32, 16), mfma(api, c.cls, 32, 64, tk, 16, 32, 16, split_k=3)], seed=n)


def test_gemv_sketch_resnet_classifier(api, P):
    k = wl.resnet18_kernels()[-1]
    assert k.gemm_extents() == (1, 1, 1000, 512)
    gemv = lambda tm, tn, wn, tk, vec: api.make_schedule(k.cls, api.TT_SK_GEMV, tm, tn, tk, tm, wn, 0, 1, 0, vec, 1, 1)
    P.check_kernel(k, [None, gemv(1, 4, 1, 256, 4), gemv(1, 8, 2, 512, 4), gemv(1, 16, 4, 64, 1), gemv(1, 2, 2, 128, 2)])
    k4 = wl.Kernel(wl.CLS_DENSE_BIAS_GELU, wl.GemmShape(1, 5, 70, 200, 1, wl.BF16), 1, "gemv_bf16")
    gemv4 = lambda tm, tn, wn, tk, vec: api.make_schedule(k4.cls, api.TT_SK_GEMV, tm, tn, tk, tm, wn, 0, 1, 0, vec, 1, 1)
    P.check_kernel(k4, [None, gemv4(2, 8, 2, 128, 8), gemv4(4, 4, 4, 64, 1)])


def test_batch_matmul_both_layouts(api, P):
    for trans_b in (1, 0):
        for dt in (wl.BF16, wl.F32):
            k = wl.Kernel(wl.CLS_BATCH_MATMUL, wl.GemmShape(5, 128, 72, 96, trans_b, dt), 1, f"bmm_t{trans_b}_{dt}")
            tk = 16 if dt == wl.F32 else 32
            scheds = [None, mfma(api, k.cls, 64, 64, tk, 32, 32, 32), mfma(api, k.cls, 32, 32, tk * 2, 16, 16, 16, split_k=2, order=4),
                      api.make_schedule(k.cls, api.TT_SK_DIRECT, 1, 1, 1, 1, 1, 0, 1, 0, 1, 1, 1)]
            P.check_kernel(k, scheds)


def test_bert_shaped_kernels_bf16(api, P):
    for k in wl.bert_kernels(seq=128, batch=2):
        scheds = [None, mfma(api, k.cls, 128, 128, 64, 64, 64, 32), mfma(api, k.cls, 64, 64, 32, 32, 32, 16, split_k=2)]
        if k.gemm_extents()[2] < 128:
            scheds[1] = mfma(api, k.cls, 64, 64, 64, 32, 32, 32)
        P.check_kernel(k, scheds)


# ---- depthwise --------------------------------------------------------------------------------------
def test_depthwise_shapes_and_records(api, P):
    dw = lambda tm, tn, tk, wm, wn, stages=1, vec=4, unroll=8, order=0: api.make_schedule(
        wl.CLS_DWCONV_BIAS_RELU6, api.TT_SK_DWCONV, tm, tn, tk, wm, wn, 0, 1, order, vec, unroll, stages)
    direct = api.make_schedule(wl.CLS_DWCONV_BIAS_RELU6, api.TT_SK_DIRECT, 1, 1, 1, 1, 1, 0, 1, 0, 1, 1, 1)
    for n, c, hw, st in ((2, 32, 112, 1), (1, 96, 112, 2), (2, 144, 56, 2), (3, 192, 28, 1), (2, 576, 14, 2), (4, 960, 7, 1)):
        k = wl.Kernel(wl.CLS_DWCONV_BIAS_RELU6, wl.ConvShape(n, c, hw, hw, c, 3, 3, st, st, 1, 1, wl.F32), 1, f"dw_{c}_{hw}_s{st}")
        ho = k.shape.ho
        scheds = [None, direct]
        if ho >= 28:
            scheds += [dw(4, 28, 4, 1, 4), dw(8, 16, 2, 2, 1, stages=2), dw(2, 28, 8, 2, 7, stages=2, order=3),
                       dw(4, 8, 8, 4, 2, unroll=1)]
        if ho >= 7:
            scheds += [dw(7, 7, 16, 1, 1), dw(7, 7, 64, 7, 1, stages=2), dw(4, 4, 16, 2, 2)]
        P.check_kernel(k, scheds)


def test_depthwise_channel_vectors_and_general_kernel(api, P):
    dw = lambda tm, tn, tk, wm, wn, stages=1, vec=4, unroll=8, order=0: api.make_schedule(
        wl.CLS_DWCONV_BIAS_RELU6, api.TT_SK_DWCONV, tm, tn, tk, wm, wn, 0, 1, order, vec, unroll, stages)
    cases = [((2, 6, 20, 20, 1, 1), 2),     # 6 channels: pairs of planes per lane
             ((3, 5, 17, 13, 2, 2), 1),     # 5 channels: one plane per lane; odd map, stride 2
             ((2, 24, 19, 19, 1, 1), 4),    # four planes per lane, ragged rows and columns
             ((1, 16, 21, 21, 3, 3), 1),    # stride 3: the general kernel, nothing vectorised
             ((2, 8, 18, 18, 2, 1), 1)]     # unequal strides: the general kernel
    for (n, c, h, w, sh, sw), want_vec in cases:
        k = wl.Kernel(wl.CLS_DWCONV_BIAS_RELU6, wl.ConvShape(n, c, h, w, c, 3, 3, sh, sw, 1, 1, wl.F32), 1, f"dw_{c}_{h}_{sh}{sw}")
        scheds = [None, dw(2, 4, 8, 1, 2), dw(4, 2, 8, 2, 1, unroll=1), dw(1, 4, 16, 1, 4, vec=2), dw(2, 2, 16, 2, 2, stages=2),
                  dw(7, 1, 64, 7, 1, vec=1)]
        plan = api.tt_schedule_apply(scheds[1], k.cls, k.shape)
        if plan.status == api.TT_OK:
            assert plan.eff_vec_a == want_vec, (k.name, plan.eff_vec_a)
            assert plan.tile_k == 8 * want_vec
        P.check_kernel(k, scheds, seed=91)


# ---- split reduction ---------------------------------------------------------------------------------
def test_split_k_is_deterministic(api, P):
    """Partial sums are added in split order by the reduce kernel: bits do not depend on scheduling."""
    from paper_2201_05587_amd import harness
    for dt in (wl.F32, wl.BF16):
        tk = 16 if dt == wl.F32 else 32
        k = conv_kernel(wl.CLS_CONV2D_BIAS_ADD_RELU, 2, 64, 14, 96, 3, 1, dtype=dt)     # K = 576, ragged N tiles
        recs = [mfma(api, k.cls, 32, 32, tk, 16, 16, 16, split_k=6), mfma(api, k.cls, 64, 64, tk, 32, 32, 16, split_k=6, stages=3),
                mfma(api, k.cls, 64, 64, tk, 32, 16, 16, split_k=6, order=4)]
        ref, outs = P.check_kernel(k, recs, seed=5)
        # the same (tile_k, split_k, matrix-core block) gives the same summation order whatever the tile, pipeline or raster
        np.testing.assert_array_equal(outs[0], outs[1])
        np.testing.assert_array_equal(outs[0], outs[2])
        dk = harness.device_kernel(k, 5)
        first = P.run_gpu(k, dk, recs[1])
        for _ in range(5):
            np.testing.assert_array_equal(P.run_gpu(k, dk, recs[1]), first)
        np.testing.assert_array_equal(first, outs[1])


# ---- kernels chained through shared tensors ---------------------------------------------------------
def test_bottleneck_chain_matches_the_oracle_applied_in_sequence(api, P):
    """Three kernels per block, the output tensor of one being the input of the next, two blocks."""
    import torch
    from oracle import ops as O
    from paper_2201_05587_amd import harness
    for dt in (wl.F32, wl.BF16):
        kr = conv_kernel(wl.CLS_CONV2D_BIAS_RELU, 2, 64, 10, 32, 1, 1, dtype=dt)
        kc = conv_kernel(wl.CLS_CONV2D_BIAS_RELU, 2, 32, 10, 32, 3, 1, dtype=dt)
        ke = conv_kernel(wl.CLS_CONV2D_BIAS_ADD_RELU, 2, 32, 10, 64, 1, 1, dtype=dt)
        dks, kinds, host = harness.bottleneck_chain(kr, kc, ke, 2, seed=17)
        tk = 16 if dt == wl.F32 else 32
        recs = [None, mfma(api, kc.cls, 32, 32, tk, 16, 16, 16, stages=3), mfma(api, ke.cls, 64, 32, tk, 32, 32, 32, split_k=2 if dt == wl.F32 else 1)] * 2
        api.KernelList(dks, recs).run(1)
        torch.cuda.synchronize()
        x = host["x0"]
        rnd = (lambda a: a) if dt == wl.F32 else O.round_to_bf16   # each kernel stores bf16 outputs
        for _ in range(2):
            y1 = rnd(O.conv2d(x, host["reduce"]["w"], host["reduce"]["bias"], None, (1, 1), (0, 0), O.ACT_RELU))
            y2 = rnd(O.conv2d(y1, host["conv"]["w"], host["conv"]["bias"], None, (1, 1), (1, 1), O.ACT_RELU))
            x = rnd(O.conv2d(y2, host["expand"]["w"], host["expand"]["bias"], x, (1, 1), (0, 0), O.ACT_RELU))
        got = harness.output_in_definition_order(ke, dks[-1].output()).float().cpu().numpy()
        # six kernels deep: the bf16 roundings of the intermediate tensors can differ by one unit in the last place
        P.assert_close(got, x, dt, f"chain {dt}")


# ---- error behaviour --------------------------------------------------------------------------------
def test_invalid_records_return_errors_and_write_nothing(api, P):
    import torch
    from paper_2201_05587_amd import harness
    k = wl.resnet18_kernels()[13]  # 7x7 maps: M = 49
    dk = harness.device_kernel(k, 5)
    dk.output().fill_(7.0)
    too_big = mfma(api, k.cls, 64, 64, 32, 32, 32, 32)
    assert dk.run(too_big) == api.TT_ERR_INVALID_SCHEDULE
    other = mfma(api, wl.CLS_CONV2D_ADD, 32, 32, 32, 16, 16, 16)
    assert dk.run(other) == api.TT_ERR_CLASS_MISMATCH
    malformed = mfma(api, k.cls, 32, 32, 32, 48, 16, 16)
    assert dk.run(malformed) == api.TT_ERR_BAD_ARG
    k2 = conv_kernel(k.cls, 1, 64, 14, 256, 3, 1)       # M = 196, N = 256
    dk2 = harness.device_kernel(k2, 6)
    dk2.output().fill_(7.0)
    no_variant = mfma(api, k.cls, 128, 256, 32, 128, 32, 32)  # well-formed, applies, but is not compiled
    assert api.tt_schedule_apply(no_variant, k2.cls, k2.shape).status == api.TT_OK
    assert dk2.run(no_variant) == api.TT_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((dk2.output() == 7.0).all())
    # split-K without enough workspace
    dk.desc.ws_bytes = 16
    assert dk.run(mfma(api, k.cls, 32, 32, 32, 16, 16, 16, split_k=4)) == api.TT_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((dk.output() == 7.0).all())
    # residual class without a residual tensor, misaligned pointer
    x = dk.tensors["x"]
    rc = api.lib.tt_conv2d_bias_relu(x.data_ptr() + 4, dk.desc.bufs[1], dk.desc.bufs[2], dk.desc.bufs[3], dk.desc.bufs[4],
                                     __import__("ctypes").byref(dk.cshape), k.cls, None, None, 0, None)
    assert rc == api.TT_ERR_BAD_ARG


def test_degenerate_shapes_fall_back_to_the_direct_or_gemv_sketch(api, P):
    """Extents too small for a matrix-core tile: the default record is the unscheduled loop nest (or GEMV)."""
    cases = [wl.Kernel(wl.CLS_CONV2D_BIAS_RELU, wl.ConvShape(1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, wl.F32), 1, "conv_1x1x1"),
             wl.Kernel(wl.CLS_CONV2D_BIAS_ADD_RELU, wl.ConvShape(2, 3, 5, 4, 7, 3, 3, 2, 1, 1, 2, wl.BF16), 1, "conv_tiny_bf16"),
             wl.Kernel(wl.CLS_DENSE_BIAS_GELU, wl.GemmShape(1, 1, 1, 1, 1, wl.F32), 1, "dense_1x1x1"),
             wl.Kernel(wl.CLS_DENSE_ADD, wl.GemmShape(1, 3, 5, 7, 1, wl.BF16), 1, "dense_tiny_bf16"),
             wl.Kernel(wl.CLS_BATCH_MATMUL, wl.GemmShape(3, 2, 3, 4, 0, wl.F32), 1, "bmm_tiny_nn"),
             wl.Kernel(wl.CLS_DWCONV_BIAS_RELU6, wl.ConvShape(1, 3, 4, 5, 3, 3, 3, 1, 1, 1, 1, wl.F32), 1, "dw_tiny")]
    for k in cases:
        rec = api.tt_schedule_default(k.cls, k.shape)
        assert rec.sketch in (api.TT_SK_DIRECT, api.TT_SK_GEMV), (k.name, rec)
        P.check_kernel(k, [None], seed=3)


def test_tensors_of_two_gib_are_refused_by_the_matrix_core_conv_not_launched(api, P):
    """The conv kernels address tensors with 32-bit byte offsets: larger ones are TT_ERR_UNSUPPORTED."""
    import ctypes
    import torch
    dummy = torch.zeros(64, device="cuda")
    huge = api.to_c_shape(wl.ConvShape(64, 256, 512, 512, 64, 3, 3, 1, 1, 1, 1, wl.BF16))   # 8 GiB of activations
    rec = mfma(api, wl.CLS_CONV2D_BIAS_RELU, 64, 64, 32, 32, 32, 16)
    assert api.tt_schedule_apply(rec, wl.CLS_CONV2D_BIAS_RELU, huge).status == api.TT_OK
    p = dummy.data_ptr()
    rc = api.lib.tt_conv2d_bias_relu(p, p, p, None, p, ctypes.byref(huge), wl.CLS_CONV2D_BIAS_RELU, ctypes.byref(rec), None, 0, None)
    assert rc == api.TT_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert float(dummy.abs().sum()) == 0.0


# ---- sweep ------------------------------------------------------------------------------------------
def test_transfer_sweep_on_cfg1(api, P):
    from paper_2201_05587_amd import harness
    target, donor = wl.cfg1_target(), wl.cfg1_donor()
    E = target.cls
    pool = [mfma(api, E, 32, 32, 32, 16, 16, 16), mfma(api, E, 64, 64, 32, 32, 32, 32), mfma(api, E, 128, 64, 32, 64, 32, 32),
            mfma(api, E, 128, 128, 32, 64, 64, 32),
            mfma(api, wl.CLS_CONV2D_ADD, 32, 32, 32, 16, 16, 16),          # other class: never tried
            mfma(api, E, 64, 64, 32, 32, 32, 32, split_k=32)]              # 18 K tiles: invalid
    dks = [harness.device_kernel(target, 11), harness.device_kernel(donor, 12)]
    rows, table, evals, wall = api.tt_transfer_sweep(dks, pool, api.make_opts(warmup=1, samples=5))
    assert evals == 2 * (1 + 5)
    for r, t in zip(rows, table):
        assert t[4] == -2.0 and r["n_other_class"] == 1
        valid = [v for i, v in enumerate(t) if i != 4 and v >= 0]
        assert r["n_valid"] == len(valid) and r["n_invalid"] == 5 - len(valid)
        assert r["best_us"] == min(valid + [r["default_us"]])
        assert all(v > 0 for v in valid) and r["default_us"] > 0
        if r["chosen"] >= 0:
            assert t[r["chosen"]] == r["best_us"] < r["default_us"]
    assert table[0][5] == -1.0          # split_k = 32 > 18 K tiles on the target
    assert table[1][5] >= 0             # but fine on the donor (36 K tiles)
    assert wall > 0
    # the chosen record still computes the right thing
    chosen = rows[0]["chosen"]
    P.check_kernel(target, [pool[chosen] if chosen >= 0 else None], seed=11)


def test_budgeted_sweep_evaluates_the_planned_pairs_only(api, P):
    """A pair budget: every default is timed, then exactly the pairs tt_sweep_plan selects (the oracle's rule)."""
    from paper_2201_05587_amd import harness
    target, donor = wl.cfg1_target(), wl.cfg1_donor()
    E = target.cls
    pool = [mfma(api, E, 32, 32, 32, 16, 16, 16), mfma(api, E, 64, 64, 32, 32, 32, 32), mfma(api, E, 128, 64, 32, 64, 32, 32),
            mfma(api, wl.CLS_CONV2D_ADD, 32, 32, 32, 16, 16, 16), mfma(api, E, 64, 32, 32, 32, 32, 16),
            mfma(api, E, 32, 64, 32, 32, 32, 16)]
    dks = [harness.device_kernel(target, 11), harness.device_kernel(donor, 12)]
    for prio in (0, 1):
        rows, table, evals, _ = api.tt_transfer_sweep(dks, pool, api.make_opts(warmup=1, samples=3, pair_budget=4,
                                                                               prioritise=prio, seed=99))
        assert evals == 2 + 4
        weights = [r["default_us"] * 1 for r in rows]
        want = S.sweep_plan([E, E], weights, [p.cls for p in pool], 4, bool(prio), 99)
        for k in range(2):
            for p in range(len(pool)):
                if pool[p].cls != E:
                    assert table[k][p] == -2.0
                elif want[k][p]:
                    assert table[k][p] > 0 or table[k][p] == -1.0
                else:
                    assert table[k][p] == -3.0
            assert rows[k]["n_not_tried"] == sum(1 for p in range(len(pool)) if pool[p].cls == E and not want[k][p])
            tried = [table[k][p] for p in range(len(pool)) if table[k][p] > 0]
            assert rows[k]["best_us"] == min(tried + [rows[k]["default_us"]])


def test_refinement_and_native_sweep_return_records_that_compute_the_operator(api, P):
    from paper_2201_05587_amd import harness
    k = conv_kernel(wl.CLS_CONV2D_BIAS_RELU, 2, 64, 28, 64, 3, 1, dtype=wl.BF16)
    dk = harness.device_kernel(k, 5, max_split=8)
    base = mfma(api, k.cls, 32, 32, 32, 16, 16, 16, stages=2)
    quick = api.make_opts(warmup=1, samples=3, min_sample_us=50, max_launches=8)
    rc, best, best_us, base_us, tried = api.tt_refine(dk, base, 2, quick)
    assert rc == api.TT_OK and 0 < best_us <= base_us and tried >= 10
    near = [r.knobs() for r in api.tt_refine_space(base)]
    assert best.knobs() == base.knobs() or best_us < base_us
    if best.knobs() != base.knobs() and best.knobs() not in near:
        # two rounds: a neighbour of a neighbour
        assert any(best.knobs() in [q.knobs() for q in api.tt_refine_space(api.make_schedule(**n))] for n in near)
    # a base that does not apply is refused, nothing timed
    bad = mfma(api, k.cls, 256, 256, 32, 64, 64, 16)
    assert api.tt_refine(dk, bad, 1, quick)[0] == api.TT_ERR_INVALID_SCHEDULE
    nbest, nbest_us, default_us, n_valid, n_rec = api.tt_native_sweep(dk, 0, 3, quick, quick)
    assert 0 < nbest_us <= default_us and 0 < n_valid <= n_rec
    plan = api.tt_schedule_apply(nbest, k.cls, k.shape)
    assert plan.status == api.TT_OK and plan.variant_id >= 0
    P.check_kernel(k, [best, nbest], seed=5)


# ---- 3x3 convolutions with the padded input patch in LDS (stages 5 and 6) ---------------------------
PATCH_CASES = [
    # (n, c, hw, k, stride), (tile_m, tile_n, tile_k, wave_m, wave_n), split_k, stages
    ((2, 64, 28, 128, 1), (128, 128, 64, 64, 64), 1, 5),      # one channel slice, tiles cross image rows
    ((3, 128, 14, 128, 1), (128, 128, 64, 64, 64), 1, 6),     # two slices, tiles cross images, ragged last tile (588 rows)
    ((3, 128, 14, 128, 1), (128, 128, 64, 64, 64), 2, 5),     # the reduction split on the slice boundary
    ((5, 256, 7, 192, 1), (128, 64, 64, 64, 32), 1, 5),       # 7 x 7 maps: a tile spans three images; ragged M (245) and N tiles
    ((5, 256, 7, 192, 1), (64, 64, 64, 64, 32), 4, 6),        # four slices, one per split
    ((1, 64, 224, 64, 1), (128, 64, 64, 64, 32), 1, 5),       # wide maps: the patch of a tile does not fit the buffer -> ring
    ((2, 64, 56, 64, 1), (128, 64, 64, 64, 32), 1, 6),
    ((1, 128, 20, 64, 1), (64, 64, 64, 64, 32), 1, 5),        # 20 x 20: rows that are no multiple of anything
    ((2, 64, 28, 128, 2), (128, 128, 32, 64, 64), 1, 5),      # stride 2: 28 -> 14
    ((4, 96, 14, 128, 2), (64, 128, 32, 64, 64), 3, 6),       # stride 2 on 14 -> 7, three slices of 32, one per split
    ((2, 64, 27, 64, 2), (64, 64, 32, 64, 32), 1, 5),         # odd input size under stride 2
    ((2, 128, 12, 256, 1), (64, 128, 64, 32, 64), 1, 5),      # wave tile split along the columns
    ((2, 64, 30, 128, 1), (256, 64, 64, 64, 64), 1, 5),
]


@pytest.mark.parametrize("case", PATCH_CASES)
@pytest.mark.parametrize("cls", [wl.CLS_CONV2D_BIAS_RELU, wl.CLS_CONV2D_BIAS_ADD_RELU])
def test_conv3x3_with_the_input_patch_in_lds(api, P, case, cls):
    (n, c, hw, kk, st), (tm, tn, tk, wm, wn), split, stages = case
    k = conv_kernel(cls, n, c, hw, kk, 3, st, dtype=wl.BF16)
    rec = mfma(api, cls, tm, tn, tk, wm, wn, 32, split_k=split, order=(stages + split) % 6, stages=stages)
    plan = api.tt_schedule_apply(rec, k.cls, k.shape)
    assert plan.status == api.TT_OK and plan.variant_id >= 0, (plan.status, plan.reason)
    P.check_kernel(k, [rec], seed=505 + stages)


def test_patch_kernel_is_the_one_that_runs_where_it_applies(api):
    """The cases above exercise the patch kernel (pipeline 2), except the one built to overflow its buffer."""
    ran = []
    for (n, c, hw, kk, st), (tm, tn, tk, wm, wn), split, stages in PATCH_CASES:
        k = conv_kernel(wl.CLS_CONV2D_BIAS_RELU, n, c, hw, kk, 3, st, dtype=wl.BF16)
        rec = mfma(api, k.cls, tm, tn, tk, wm, wn, 32, split_k=split, stages=stages)
        plan = api.tt_schedule_apply(rec, k.cls, k.shape)
        ran.append(api.tt_variant_info(plan.variant_id)[9])
    assert ran.count(2) == len(PATCH_CASES) - 1 and ran[5] == 1


# ---- persistent kernel of the dense family: B panel resident in LDS (stages 7) ------------------------
STREAM_CASES = [
    # kernel, (tile_m, tile_n, tile_k, wave_m, wave_n, mfma)
    # 1x1 convolution with residual, one slice; 1568 tiles for 512 resident workgroups: three tiles each
    (wl.Kernel(wl.CLS_CONV2D_BIAS_ADD_RELU, wl.ConvShape(16, 64, 56, 56, 256, 1, 1, 1, 1, 0, 0, wl.BF16), 1, "pw_res"),
     (64, 128, 64, 32, 64, 32)),
    # ragged M (1 x 37 x 37 = 1369 rows) and a ragged last panel (N = 200), two slices, 16-blocks
    (wl.Kernel(wl.CLS_CONV2D_BIAS_RELU, wl.ConvShape(1, 128, 37, 37, 200, 1, 1, 1, 1, 0, 0, wl.BF16), 1, "pw_ragged"),
     (64, 128, 64, 32, 64, 16)),
    # fewer tiles than resident workgroups: some workgroups get one tile, the loop of none runs twice
    (wl.Kernel(wl.CLS_DENSE_BIAS_GELU, wl.GemmShape(1, 300, 256, 256, 1, wl.BF16), 1, "dense_few_tiles"),
     (32, 128, 64, 32, 32, 16)),
    # four slices of 64, linear epilogue, rows that are not whole vectors long (N = 70: element path)
    (wl.Kernel(wl.CLS_DENSE_ADD, wl.GemmShape(1, 5000, 70, 256, 1, wl.BF16), 1, "dense_narrow"),
     (64, 64, 64, 32, 32, 32)),
    # one-batch A.B^T product, no bias at all
    (wl.Kernel(wl.CLS_BATCH_MATMUL, wl.GemmShape(1, 2048, 384, 128, 1, wl.BF16), 1, "bmm_one_batch"),
     (128, 64, 64, 32, 32, 16)),
    # fp32: pointwise ReLU6 with ragged everything, a dense layer on eight waves, and one on 32-blocks
    (wl.Kernel(wl.CLS_CONV2D_BIAS_RELU6, wl.ConvShape(3, 96, 29, 29, 144, 1, 1, 1, 1, 0, 0, wl.F32), 1, "pw_f32"),
     (64, 128, 32, 32, 64, 16)),
    (wl.Kernel(wl.CLS_DENSE_BIAS_RELU, wl.GemmShape(1, 4100, 128, 64, 1, wl.F32), 1, "dense_f32"),
     (128, 128, 16, 32, 64, 16)),
    (wl.Kernel(wl.CLS_DENSE_BIAS_RELU, wl.GemmShape(1, 9000, 192, 64, 1, wl.F32), 1, "dense_f32_blocks32"),
     (64, 64, 32, 32, 32, 32)),
]


@pytest.mark.parametrize("case", STREAM_CASES, ids=[c[0].name for c in STREAM_CASES])
def test_persistent_dense_kernel_with_the_panel_in_lds(api, P, case):
    k, (tm, tn, tk, wm, wn, mf) = case
    vec = 8 if k.shape.dtype == wl.BF16 else 4
    recs = [mfma(api, k.cls, tm, tn, tk, wm, wn, mf, order=o, vec=vec, stages=7) for o in (0, 4)]
    for rec in recs:
        plan = api.tt_schedule_apply(rec, k.cls, k.shape)
        assert plan.status == api.TT_OK and plan.stages == 7 and api.tt_variant_info(plan.variant_id)[9] == 3, \
            (plan.status, plan.reason, plan.stages, plan.variant_id)
    P.check_kernel(k, recs, seed=707)


def test_machine_rate_probes_copy_exactly_and_report_plausible_rates(api):
    """The probes are plain kernels: the copies must reproduce their source, every rate must be positive and below
    what the hardware can do, and bad arguments are refused before anything is launched."""
    import torch
    n = 64 << 20
    src = torch.arange(n // 4, dtype=torch.int32, device="cuda")
    for which in (api.TT_PROBE_COPY_LINEAR_GBPS, api.TT_PROBE_COPY_TILED_GBPS):
        dst = torch.zeros_like(src)
        gbps = api.tt_debug_probe(which, src, dst, reps=3)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
        assert 100.0 < gbps < 2.0e4, gbps
    small = torch.ones((1 << 20) // 4, dtype=torch.int32, device="cuda")
    assert 0.5 < api.tt_debug_probe(api.TT_PROBE_LAUNCH_GAP_US, reps=50) < 100.0
    assert 100.0 < api.tt_debug_probe(api.TT_PROBE_MFMA_BF16_TFLOPS, dst=small, reps=2) < 3000.0
    assert 1.0e3 < api.tt_debug_probe(api.TT_PROBE_L2_READ_GBPS, small, dst, reps=2) < 2.0e5
    odd = torch.ones(1000, dtype=torch.int32, device="cuda")
    with pytest.raises(api.TTError):
        api.tt_debug_probe(api.TT_PROBE_COPY_LINEAR_GBPS, odd, odd, reps=1)
    with pytest.raises(api.TTError):
        api.tt_debug_probe(99, src, dst, reps=1)


def test_timing_rotates_through_the_alternative_tensor_sets(api, P):
    """With alternates every launch of a timed pair takes the next tensor set: all of them end up holding the
    operator's output, and a streaming kernel timed over sets larger than the caches is not faster than on one."""
    import torch
    from paper_2201_05587_amd import harness
    k = wl.Kernel(wl.CLS_CONV2D_BIAS_ADD_RELU, wl.ConvShape(32, 64, 56, 56, 256, 1, 1, 1, 1, 0, 0, wl.BF16), 1, "rotate")
    warm = harness.device_kernel(k, 77)
    cold = harness.device_kernel(k, 77, cold_mb=700.0)
    assert len(cold.alternates) >= 6 and cold.desc.n_alt == len(cold.alternates)
    for alt in cold.alternates:
        alt["y"].fill_(float("nan"))
    opts = api.make_opts(warmup=2, samples=5, min_sample_us=300, max_launches=32)
    st_w, warm_us, _ = api.tt_time_pair(warm, None, opts)
    st_c, cold_us, _ = api.tt_time_pair(cold, None, opts)
    torch.cuda.synchronize()
    assert st_w == api.TT_OK and st_c == api.TT_OK
    for alt in cold.alternates:
        assert torch.equal(alt["y"], warm.output())
    assert torch.equal(cold.output(), warm.output())
    assert cold_us > 0.9 * warm_us, (cold_us, warm_us)
    # a descriptor that announces alternates without naming them is refused
    cold.desc.alt_bufs = None
    st, _, _ = api.tt_time_pair(cold, None, opts)
    assert st == api.TT_ERR_BAD_ARG
