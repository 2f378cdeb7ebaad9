"""Host logic of libtt against the integer oracle, bit for bit (no GPU needed)."""
import os
import random
import re

import pytest

from oracle import schedule as S
from paper_2201_05587_amd import api
from paper_2201_05587_amd import workloads as wl
from test_oracle_schedule import all_cfg_kernels, oshape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def to_c_record(rec: dict) -> api.tt_schedule:
    return api.make_schedule(**{k: rec[k] for k in S.RECORD_FIELDS})


RESOURCE_REASONS = (6, 7)  # TT_R_LDS, TT_R_K_GRANULE: the library's own, checked after every method rule


def plan_equal(cplan: api.tt_plan, oplan: dict, rec=None):
    """The method fields of the library's plan against the oracle's, bit for bit.

    Where the library rejects a record for a reason of its own kernels (LDS size, K step of the matrix
    cores) the oracle must have found the record valid as far as the method goes; the library's claim is
    then checked against what its compiled kernels export.
    """
    assert set(api.tt_plan.METHOD_FIELDS) == set(S.PLAN_FIELDS)
    if cplan.status == api.TT_ERR_INVALID_SCHEDULE and cplan.reason in RESOURCE_REASONS:
        assert oplan["status"] == S.OK, (cplan.reason, oplan)
        assert rec is not None and rec["sketch"] in (S.SK_MFMA, S.SK_DWCONV)
        if cplan.reason == 7:
            assert rec["tile_k"] % min(g for d, mf, g in kernel_k_granules() if mf == rec["mfma"]) or \
                any(rec["tile_k"] % g for d, mf, g in kernel_k_granules() if mf == rec["mfma"])
        return False
    got = cplan.method()
    diff = {k: (got[k], oplan[k]) for k in S.PLAN_FIELDS if got[k] != oplan[k]}
    assert not diff, diff
    return True


_VARIANTS = []


def all_variants():
    if not _VARIANTS:
        for i in range(api.lib.tt_num_variants()):
            _VARIANTS.append(dict(zip(api.VARIANT_INFO, api.tt_variant_info(i))))
    return _VARIANTS


def kernel_k_granules():
    """(dtype, mfma, K elements per matrix-core step) as the compiled kernels report them."""
    return sorted({(v["dtype"], v["mfma"], v["k_granule"]) for v in all_variants()})


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "tt.h")) as f:
        text = f.read()
    declared = set(re.findall(r"^(?:int|int64_t|const char \*)\s*(tt_\w+)\(", text, flags=re.M))
    assert declared == set(api.EXPORTS), declared ^ set(api.EXPORTS)
    for name in declared:
        assert hasattr(api.lib, name)
    assert api.lib.tt_version() >= 100
    assert api.status_name(-1) == "TT_ERR_INVALID_SCHEDULE"


def test_default_schedule_matches_oracle_on_every_configured_shape():
    for k in all_cfg_kernels():
        got = api.tt_schedule_default(k.cls, k.shape).knobs()
        assert got == S.default_schedule(k.cls, oshape(k)), k.name
    tiny = wl.Kernel(wl.CLS_CONV2D_BIAS_RELU, wl.ConvShape(1, 2, 4, 4, 3, 3, 3, 1, 1, 1, 1))
    assert api.tt_schedule_default(tiny.cls, tiny.shape).knobs() == S.default_schedule(tiny.cls, oshape(tiny))


def random_record(rng, cls):
    if cls == S.CLS_DWCONV_BIAS_RELU6 and rng.random() < 0.9:
        return S.record(cls, S.SK_DWCONV, rng.choice([1, 2, 4, 7, 8, 14, 16]), rng.choice([4, 7, 8, 14, 16, 28, 32, 56]),
                        rng.choice([1, 2, 4, 8, 16]), rng.choice([1, 2, 4, 7]), rng.choice([1, 2, 4, 7]), 0, 1,
                        rng.randrange(6), rng.choice([1, 2, 4, 8]), rng.choice([1, 2, 4]), rng.choice([1, 2]))
    u = rng.random()
    if u < 0.05:
        return S.record(cls, S.SK_DIRECT, 1, 1, 1, 1, 1, 0, 1, 0, 1, 1, 1)
    if u < 0.15:
        tm = rng.choice([1, 2, 4])
        wn = rng.choice([1, 2, 4])
        return S.record(cls, S.SK_GEMV, tm, wn * rng.choice([1, 2, 4, 8]), 64 * rng.choice([1, 2, 4, 8]), tm, wn, 0, 1,
                        rng.randrange(6), rng.choice([1, 2, 4, 8]), rng.choice([1, 2, 8]), 1)
    tm, tn = rng.choice([16, 32, 64, 128, 256]), rng.choice([16, 32, 64, 128, 256])
    mf = rng.choice([16, 32])
    return S.record(cls, S.SK_MFMA, tm, tn, rng.choice([16, 32, 64, 128]), rng.choice([16, 32, 64, 128]),
                    rng.choice([16, 32, 64, 128]), mf, rng.choice([1, 1, 2, 3, 4, 8, 16, 64]), rng.randrange(6),
                    rng.choice([1, 2, 4, 8]), rng.choice([1, 2, 4, 512]), rng.choice([1, 2, 3, 4, 5, 6, 7]))


def test_apply_matches_oracle_bit_for_bit_on_random_records():
    rng = random.Random(20220105)
    kernels = all_cfg_kernels()
    statuses = {}
    resource_rejections = 0
    for it in range(6000):
        k = rng.choice(kernels)
        rec = random_record(rng, k.cls if rng.random() < 0.9 else rng.randrange(S.NUM_CLASSES))
        flags = S.STRICT_DIVISIBLE if rng.random() < 0.2 else 0
        oplan = S.apply(rec, k.cls, oshape(k), flags)
        cplan = api.tt_schedule_apply(to_c_record(rec), k.cls, k.shape, flags)
        statuses[oplan["status"]] = statuses.get(oplan["status"], 0) + 1
        if not plan_equal(cplan, oplan, rec):
            resource_rejections += 1
            continue
        if oplan["status"] == S.OK:
            check_library_fields(cplan, rec, k)
        if oplan["status"] == S.OK and oplan["sketch"] != S.SK_DIRECT and oplan["grid"] <= 4096 and it % 10 == 0:
            for wg in range(oplan["grid"]):
                assert api.tt_plan_tile(cplan, wg) == S.plan_tile(oplan, wg)
    # the draw must exercise every outcome
    assert all(statuses.get(s, 0) > 50 for s in (S.OK, S.ERR_INVALID_SCHEDULE, S.ERR_CLASS_MISMATCH, S.ERR_BAD_ARG))
    assert 0 < resource_rejections < 1500


def check_library_fields(cplan, rec, k):
    """The plan fields that describe the library's kernels, against what those kernels export and against
    the properties a reformulated knob must have (Section 4.1): never wider than asked, a power of two,
    dividing the extent it runs along, and maximal."""
    s = k.shape
    widest = 4 if s.dtype == wl.F32 else 8
    if cplan.sketch == api.TT_SK_MFMA:
        if k.is_conv():
            along = dict(eff_vec_a=s.c, eff_vec_b=s.c, eff_vec_c=cplan.N)   # channels-last tensors
        else:
            along = dict(eff_vec_a=cplan.K, eff_vec_b=cplan.K if s.trans_b else cplan.N, eff_vec_c=cplan.N)
        for f, extent in along.items():
            v = getattr(cplan, f)
            assert v == S.pow2_dividing(min(rec["vec"], widest), extent), (f, v, rec["vec"], extent)
        assert 1 <= cplan.eff_unroll <= rec["unroll"]
        # reformulation chain of the cache-buffer knob: resident panel (7) -> ring of four; patch + ring (5, 6) ->
        # ring (3, 4) -> two register stages
        assert cplan.stages in {rec["stages"]} | ({4, 2} if rec["stages"] == 7 else set()) | \
            ({rec["stages"] - 2, 2} if rec["stages"] in (5, 6) else set()) | ({2} if rec["stages"] >= 3 else set())
        if cplan.variant_id >= 0:
            v = dict(zip(api.VARIANT_INFO, api.tt_variant_info(cplan.variant_id)))
            assert (v["dtype"], v["tile_m"], v["tile_n"], v["tile_k"], v["wave_m"], v["wave_n"], v["mfma"]) == \
                (s.dtype, rec["tile_m"], rec["tile_n"], rec["tile_k"], rec["wave_m"], rec["wave_n"], rec["mfma"])
            assert v["pipe"] == (3 if cplan.stages == 7 else 2 if cplan.stages >= 5 else 1 if cplan.stages >= 3 else 0)
            if v["pipe"] == 3:
                # the whole panel of B, two A buffers and the epilogue's staging; requests within the counter
                es = 4 if s.dtype == wl.F32 else 2
                assert 160 * 1024 >= cplan.lds_bytes > cplan.k_tiles * (rec["tile_n"] + 2 * rec["tile_m"]) * rec["tile_k"] * es
                assert cplan.K % rec["tile_k"] == 0 and cplan.batch == 1 and cplan.eff_split_k == 1
                assert cplan.k_tiles * v["stage_bytes"] + 8 <= 63
            elif v["pipe"] < 2:
                assert cplan.lds_bytes == cplan.stages * v["stage_bytes"] <= 160 * 1024
            else:
                # two patch buffers of the exported pixel capacity and a ring of stages - 2 filter tiles
                assert 160 * 1024 >= cplan.lds_bytes >= 2 * v["stage_bytes"] * rec["tile_k"] * 2 + \
                    (cplan.stages - 2) * rec["tile_n"] * rec["tile_k"] * 2
                assert s.c % rec["tile_k"] == 0 and cplan.k_iters % 9 == 0 and (s.r, s.s) == (3, 3)
            assert rec["tile_k"] % v["k_granule"] == 0
            assert cplan.eff_unroll == min(rec["unroll"], rec["tile_k"] // v["k_granule"])
            # a stage holds at least the two operand tiles
            assert v["pipe"] == 3 or \
                v["stage_bytes"] >= (rec["tile_m"] + rec["tile_n"]) * rec["tile_k"] * (4 if s.dtype == wl.F32 else 2)
        else:
            assert cplan.lds_bytes == 0
    elif cplan.sketch == api.TT_SK_DWCONV:
        assert cplan.eff_vec_a == S.pow2_dividing(min(rec["vec"], widest), s.c)
        assert cplan.tile_k == rec["tile_k"] * cplan.eff_vec_a
        # several planes per lane run in the one-stage kernel only; workgroups of up to 256 threads always
        # have a kernel, larger ones only where a lane's window fits the registers left to it
        kinds = cplan.eff_vec_a == 1 or rec["stages"] == 1
        if cplan.variant_id >= 0:
            assert kinds
        elif kinds:
            assert cplan.block > 256
    else:
        assert cplan.variant_id == 0


@pytest.mark.parametrize("order", range(6))
def test_plan_tile_matches_oracle_for_every_order_on_the_configured_shapes(order):
    rng = random.Random(order)
    for k in all_cfg_kernels():
        if k.cls == wl.CLS_DWCONV_BIAS_RELU6:
            rec = S.record(k.cls, S.SK_DWCONV, 4, 4, 4, 1, 1, 0, 1, order, 1, 1, 1)
        else:
            rec = S.record(k.cls, S.SK_MFMA, 32, 32, 32, 16, 16, 16, rng.choice([1, 2, 5]), order)
        oplan = S.apply(rec, k.cls, oshape(k))
        cplan = api.tt_schedule_apply(to_c_record(rec), k.cls, k.shape)
        assert plan_equal(cplan, oplan, rec)
        if oplan["status"] != S.OK:
            continue
        g = oplan["grid"]
        for wg in sorted(set(list(range(min(g, 40))) + [rng.randrange(g) for _ in range(60)] + [g - 1])):
            assert api.tt_plan_tile(cplan, wg) == S.plan_tile(oplan, wg)


def test_plan_tile_rejects_bad_arguments():
    k = wl.cfg1_target()
    plan = api.tt_schedule_apply(api.tt_schedule_default(k.cls, k.shape), k.cls, k.shape)
    with pytest.raises(api.TTError):
        api.tt_plan_tile(plan, plan.grid)
    with pytest.raises(api.TTError):
        api.tt_plan_tile(plan, -1)
    bad = api.tt_schedule_apply(api.make_schedule(k.cls, tile_m=256, tile_n=256, wave_m=64, wave_n=64), k.cls, k.shape)
    assert bad.status == api.TT_ERR_INVALID_SCHEDULE
    with pytest.raises(api.TTError):
        api.tt_plan_tile(bad, 0)
    assert api.tt_schedule_apply(None, k.cls, k.shape).status == api.TT_ERR_BAD_ARG


def test_sweep_selection_matches_oracle():
    rng = random.Random(7)
    for _ in range(200):
        nk, np_ = rng.randrange(1, 6), rng.randrange(0, 8)
        kc = [rng.randrange(3) for _ in range(nk)]
        pc = [rng.randrange(3) for _ in range(np_)]
        pair = [[rng.choice([-1.0, 1.0, 2.0, 3.0, 4.0]) for _ in range(np_)] for _ in range(nk)]
        default = [rng.choice([1.0, 2.0, 3.0]) for _ in range(nk)]
        for allow in (False, True):
            want = S.select(kc, pc, pair, default, allow)
            got = api.tt_sweep_select(kc, pc, pair, default, allow)
            assert [tuple(g) for g in got] == [tuple(w) for w in want]


def test_schedule_space_is_well_formed_and_contains_the_default_tiles():
    for cls, dt in ((wl.CLS_CONV2D_BIAS_RELU, wl.F32), (wl.CLS_DENSE_ADD, wl.BF16), (wl.CLS_BATCH_MATMUL, wl.BF16),
                    (wl.CLS_DWCONV_BIAS_RELU6, wl.F32)):
        space = api.tt_schedule_space(cls, dt, 1)
        assert len(space) > 10
        for r in space:
            assert S.record_is_well_formed(r.knobs()), r
            assert r.cls == cls
    # every tile the patch kernel is compiled for is in the space with stages 5 and 6, also where no other
    # kernel implements the tile (then with those stages only), and no record is listed twice
    space = api.tt_schedule_space(wl.CLS_CONV2D_BIAS_RELU, wl.BF16, 2)
    keys = [tuple(r.knobs().values()) for r in space]
    assert len(set(keys)) == len(keys)
    tile = lambda r: (r.tile_m, r.tile_n, r.tile_k, r.wave_m, r.wave_n, r.mfma)
    stages_of = {}
    for r in space:
        stages_of.setdefault(tile(r), set()).add(r.stages)
    patch_tiles = {tuple(v[f] for f in ("tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "mfma"))
                   for v in all_variants() if v["pipe"] == 2}
    assert len(patch_tiles) >= 8
    for t in patch_tiles:
        assert {5, 6} <= stages_of[t], t
    assert any(stages_of[t] == {5, 6} for t in patch_tiles)
    assert all(({5, 6} & st) == set() or t in patch_tiles for t, st in stages_of.items())
    # every default matrix-core record of the configured shapes has a compiled variant
    for k in all_cfg_kernels():
        rec = api.tt_schedule_default(k.cls, k.shape)
        plan = api.tt_schedule_apply(rec, k.cls, k.shape)
        assert plan.status == api.TT_OK
        assert plan.variant_id >= 0, (k.name, rec)


def test_resource_rejections_come_from_the_compiled_kernels():
    """TT_R_LDS and TT_R_K_GRANULE are decided by constants the kernels export, not by a second model."""
    vs = all_variants()
    assert len(vs) > 100
    # every compiled tile_k is a multiple of its kernel's K step; a record whose tile_k is not is refused
    assert all(v["tile_k"] % v["k_granule"] == 0 for v in vs)
    bsh = wl.Kernel(wl.CLS_DENSE_ADD, wl.GemmShape(1, 256, 256, 256, 1, wl.BF16))
    step16 = {v["k_granule"] for v in vs if v["dtype"] == wl.BF16 and v["mfma"] == 16}
    assert len(step16) == 1 and 16 % step16.pop() != 0
    p = api.tt_schedule_apply(api.make_schedule(bsh.cls, tile_k=16, mfma=16, vec=8), bsh.cls, bsh.shape)
    assert (p.status, p.reason) == (api.TT_ERR_INVALID_SCHEDULE, 7)
    assert api.tt_schedule_apply(api.make_schedule(bsh.cls, tile_k=16, mfma=32, vec=8), bsh.cls, bsh.shape).status == api.TT_OK
    # a ring tile that fits three times but not four: four stages are refused, three are a plan
    fits3 = [v for v in vs if v["dtype"] == wl.BF16 and v["family"] == 1 and v["pipe"] == 1
             and 3 * v["stage_bytes"] <= 160 * 1024 < 4 * v["stage_bytes"]]
    assert fits3
    big = fits3[0]
    wide = wl.Kernel(wl.CLS_DENSE_ADD, wl.GemmShape(1, 4096, 4096, 4096, 1, wl.BF16))
    rec = {f: big[f] for f in ("tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "mfma")}
    two = api.tt_schedule_apply(api.make_schedule(wide.cls, vec=8, stages=4, **rec), wide.cls, wide.shape)
    one = api.tt_schedule_apply(api.make_schedule(wide.cls, vec=8, stages=3, **rec), wide.cls, wide.shape)
    assert (two.status, two.reason) == (api.TT_ERR_INVALID_SCHEDULE, 6)
    assert one.status == api.TT_OK and one.lds_bytes == 3 * big["stage_bytes"]
    # the method still accepts both: the oracle knows nothing of LDS
    orec = S.record(wide.cls, vec=8, stages=4, **rec)
    assert S.apply(orec, wide.cls, oshape(wide))["status"] == S.OK


def test_depthwise_workgroup_size_is_limited_by_the_window_a_lane_holds():
    """A workgroup of more than 512 threads leaves a lane 128 registers: the widest windows have no kernel there, the
    method accepts the record all the same, and at 256 threads every window has one."""
    dw = wl.Kernel(wl.CLS_DWCONV_BIAS_RELU6, wl.ConvShape(1, 128, 56, 56, 128, 3, 3, 2, 2, 1, 1))
    for tile_k, tile_m, expect in ((8, 28, -1), (8, 8, 0)):
        rec = dict(sketch=api.TT_SK_DWCONV, tile_m=tile_m, tile_n=28, tile_k=tile_k, wave_m=1, wave_n=7, mfma=0,
                   vec=4, stages=1)
        p = api.tt_schedule_apply(api.make_schedule(dw.cls, **rec), dw.cls, dw.shape)
        assert p.status == api.TT_OK and p.block == tile_k * tile_m * 4 and p.variant_id == expect, (p.block, p.variant_id)
        assert S.apply(S.record(dw.cls, S.SK_DWCONV, tile_m, 28, tile_k, 1, 7, 0, 1, 0, 4, 1, 1), dw.cls, oshape(dw))["status"] == S.OK
    narrow = dict(sketch=api.TT_SK_DWCONV, tile_m=28, tile_n=4, tile_k=8, wave_m=1, wave_n=1, mfma=0, vec=1, stages=1)
    p = api.tt_schedule_apply(api.make_schedule(dw.cls, **narrow), dw.cls, dw.shape)
    assert p.status == api.TT_OK and p.block == 896 and p.variant_id == 0


def test_ring_stages_are_reformulated_where_no_ring_kernel_applies():
    bf = wl.BF16
    E = wl.CLS_CONV2D_BIAS_RELU
    conv = wl.ConvShape(32, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, bf)
    rec = dict(tile_m=64, tile_n=64, tile_k=64, wave_m=32, wave_n=32, mfma=32, vec=8, unroll=8)
    p = api.tt_schedule_apply(api.make_schedule(E, stages=4, **rec), E, conv)
    info = dict(zip(api.VARIANT_INFO, api.tt_variant_info(p.variant_id)))
    assert (p.status, p.stages, info["pipe"], p.lds_bytes) == (api.TT_OK, 4, 1, 4 * info["stage_bytes"])
    # a narrower vector knob gathers element by element: no ring, two stages of the register pipeline
    p = api.tt_schedule_apply(api.make_schedule(E, stages=4, **dict(rec, vec=4)), E, conv)
    assert p.stages == 2 and api.tt_variant_info(p.variant_id)[9] == 0
    # 3 input channels never fill an item
    stem = wl.ConvShape(32, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3, bf)
    assert api.tt_schedule_apply(api.make_schedule(E, stages=4, **rec), E, stem).stages == 2
    # the [K][N] operand of a non-transposed batch matmul stays on the register pipeline
    bm = wl.CLS_BATCH_MATMUL
    assert api.tt_schedule_apply(api.make_schedule(bm, stages=3, **rec), bm, wl.GemmShape(4, 128, 128, 64, 0, bf)).stages == 2
    assert api.tt_schedule_apply(api.make_schedule(bm, stages=3, **rec), bm, wl.GemmShape(4, 128, 128, 64, 1, bf)).stages == 3
    # eight stages is not a record
    assert api.tt_schedule_apply(api.make_schedule(E, stages=8, **rec), E, conv).status == api.TT_ERR_BAD_ARG


def test_resident_panel_stage_applies_to_short_dense_reductions_and_is_reformulated_elsewhere():
    bf = wl.BF16
    E, D = wl.CLS_CONV2D_BIAS_RELU, wl.CLS_DENSE_ADD
    rec = dict(tile_m=64, tile_n=128, tile_k=64, wave_m=32, wave_n=64, mfma=32, vec=8, unroll=8)
    pipe = lambda p: api.tt_variant_info(p.variant_id)[9]
    # a unit-stride 1x1 convolution is a dense product: K = 64 is one slice
    pw = wl.ConvShape(32, 64, 56, 56, 256, 1, 1, 1, 1, 0, 0, bf)
    p = api.tt_schedule_apply(api.make_schedule(E, stages=7, **rec), E, pw)
    assert (p.status, p.stages, pipe(p), p.k_tiles) == (api.TT_OK, 7, 3, 1) and 0 < p.lds_bytes <= 160 * 1024
    # the method part of the plan does not depend on the stage knob
    q = api.tt_schedule_apply(api.make_schedule(E, stages=4, **rec), E, pw)
    assert p.method() == q.method() and (q.stages, pipe(q)) == (4, 1)
    # a 3x3 filter, a stride, a split reduction, several batches, a K that is not whole slices, a K too long for
    # the LDS: the ring of four (or what the ring falls back to)
    for cls, shape, extra in ((E, wl.ConvShape(32, 64, 56, 56, 256, 3, 3, 1, 1, 1, 1, bf), {}),
                              (E, wl.ConvShape(32, 64, 56, 56, 256, 1, 1, 2, 2, 0, 0, bf), {}),
                              (D, wl.GemmShape(1, 4096, 256, 128, 1, bf), dict(split_k=2)),
                              (wl.CLS_BATCH_MATMUL, wl.GemmShape(4, 4096, 256, 64, 1, bf), {}),
                              (D, wl.GemmShape(1, 4096, 256, 96, 1, bf), {}),
                              (D, wl.GemmShape(1, 4096, 256, 1024, 1, bf), {})):
        p = api.tt_schedule_apply(api.make_schedule(cls, stages=7, **dict(rec, **extra)), cls, shape)
        assert p.status == api.TT_OK and p.stages in (4, 2) and pipe(p) in (0, 1), (shape, p.stages)
    # dense and one-batch A.B^T products qualify
    for cls, shape in ((D, wl.GemmShape(1, 4096, 256, 128, 1, bf)), (wl.CLS_BATCH_MATMUL, wl.GemmShape(1, 4096, 256, 64, 1, bf))):
        p = api.tt_schedule_apply(api.make_schedule(cls, stages=7, **rec), cls, shape)
        assert (p.status, p.stages, pipe(p)) == (api.TT_OK, 7, 3)
    # the oracle accepts the record like any other stage count
    assert S.apply(S.record(D, S.SK_MFMA, 64, 128, 64, 32, 64, 32, 1, 0, 8, 8, 7), D, oshape(wl.Kernel(D, wl.GemmShape(1, 4096, 256, 128, 1, bf))))["status"] == S.OK


def test_patch_stages_apply_to_3x3_bf16_convolutions_and_are_reformulated_elsewhere():
    bf = wl.BF16
    E = wl.CLS_CONV2D_BIAS_RELU
    rec = dict(tile_m=128, tile_n=128, tile_k=64, wave_m=64, wave_n=64, mfma=32, vec=8, unroll=8)
    s3 = wl.ConvShape(32, 256, 14, 14, 256, 3, 3, 1, 1, 1, 1, bf)
    p = api.tt_schedule_apply(api.make_schedule(E, stages=5, **rec), E, s3)
    info = dict(zip(api.VARIANT_INFO, api.tt_variant_info(p.variant_id)))
    assert (p.status, p.stages, info["pipe"]) == (api.TT_OK, 5, 2) and p.block == 256  # wave positions; two waves each
    # 128 consecutive output pixels of 14 x 14 maps: at most 10 rows of 16 padded pixels plus the two-row,
    # two-column halo, and one more row pair where the run crosses into the next image
    assert 200 <= info["stage_bytes"]
    assert api.tt_schedule_apply(api.make_schedule(E, stages=6, **rec), E, s3).stages == 6
    # a split of the reduction on a channel-slice boundary keeps the patch kernel (4 slices: 2 + 2) ...
    p = api.tt_schedule_apply(api.make_schedule(E, stages=5, split_k=2, **rec), E, s3)
    assert (p.stages, p.k_iters, p.eff_split_k) == (5, 18, 2)
    # ... one that cuts through a slice's nine taps falls back to the ring (36 K tiles in 3 splits of 12)
    p = api.tt_schedule_apply(api.make_schedule(E, stages=5, split_k=3, **rec), E, s3)
    assert (p.stages, p.k_iters) == (3, 12) and api.tt_variant_info(p.variant_id)[9] == 1
    # 1x1 filters, fp32, 16-blocks, 96 channels (64 does not divide them): the ring, or two stages where there is none
    pw = wl.ConvShape(32, 256, 14, 14, 256, 1, 1, 1, 1, 0, 0, bf)
    assert api.tt_schedule_apply(api.make_schedule(E, stages=6, **rec), E, pw).stages == 4
    f32 = wl.ConvShape(4, 256, 14, 14, 256, 3, 3, 1, 1, 1, 1, wl.F32)
    assert api.tt_schedule_apply(api.make_schedule(E, stages=5, **dict(rec, tile_k=32, vec=4)), E, f32).stages in (2, 3)
    c96 = wl.ConvShape(32, 96, 14, 14, 256, 3, 3, 1, 1, 1, 1, bf)
    assert api.tt_schedule_apply(api.make_schedule(E, stages=5, **rec), E, c96).stages == 3
    # a patch that does not fit the kernel's buffer: 128 output pixels of a 112-wide map under stride 2
    wide = wl.ConvShape(2, 64, 224, 224, 128, 3, 3, 2, 2, 1, 1, bf)
    p = api.tt_schedule_apply(api.make_schedule(E, stages=5, **dict(rec, tile_k=32)), E, wide)
    assert p.status == api.TT_OK and p.stages == 3
    # the method's fields do not depend on the knob
    for st in (2, 4, 6):
        o = S.apply(S.record(E, stages=st, **rec), E, oshape(wl.Kernel(E, s3)))
        c = api.tt_schedule_apply(api.make_schedule(E, stages=st, **rec), E, s3)
        assert plan_equal(c, o, S.record(E, stages=st, **rec))


def test_division_by_multiplication_is_exact():
    """The kernels turn a pixel index into (image, row, column) with a multiply; it must equal n // d."""
    import random
    from paper_2201_05587_amd import api
    rnd = random.Random(5)
    top = 2 ** 31 - 1
    ds = list(range(1, 300)) + [7 * 7, 14 * 14, 56 * 56, 112 * 112, 2 ** 16, 2 ** 16 + 1, 2 ** 30, 2 ** 30 + 1, top]
    ds += [rnd.randrange(1, top) for _ in range(300)]
    for d in ds:
        ns = [0, 1, d - 1, d, d + 1, top, top - 1, (top // d) * d, max((top // d) * d - 1, 0)]
        ns += [rnd.randrange(0, top) for _ in range(40)] + [k * d - 1 for k in range(1, 40) if k * d - 1 <= top]
        for n in ns:
            if n > top:
                continue
            assert api.lib.tt_debug_fast_div(n, d) == n // d, (n, d)
    assert api.lib.tt_debug_fast_div(5, 0) == -1 and api.lib.tt_debug_fast_div(2 ** 31, 3) == -1


def test_donor_model_selection_matches_the_oracle_and_the_papers_choices():
    """Eq. 1 in the library against the integer/float oracle and against Table 2's "Tuning Model" column."""
    from test_oracle_schedule import parse_table2
    models, _, _, _ = parse_table2()
    classes = sorted({c for m in models.values() for c in m["cls"]})
    for mid, m in models.items():
        others = [t for t in models if t != mid]
        cost = [m["cls"].get(c, (0, 0.0))[1] for c in classes]           # per cent of untuned time, any scale
        counts = [[models[t]["cls"].get(c, (0, 0.0))[0] for c in classes] for t in others]
        best, scores = api.tt_select_donor(cost, counts)
        total = sum(cost)
        want = [S.model_selection_score({c: p / total for c, p in zip(classes, cost)}, dict(zip(classes, row)))
                for row in counts]
        assert all(abs(a - b) <= 1e-12 * max(1.0, abs(b)) for a, b in zip(scores, want))
        # the oracle's choice, ties to the lowest index; where the paper's percentages add to 100 it is Table 2's model
        assert best == max(range(len(want)), key=lambda i: (want[i], -i))
        assert others[best] == m["tuning"], (mid, others[best])
    assert api.tt_select_donor([1.0, 2.0], []) == (-1, [])
    with pytest.raises(api.TTError):
        api.tt_select_donor([0.0, 0.0], [[1, 1]])
    with pytest.raises(api.TTError):
        api.tt_select_donor([1.0, 1.0], [[1, -1]])


def test_choose_donor_pool_on_the_committed_sweep_outcomes():
    """Eq. 1 end to end on stored data: ResNet18's default timings against the four committed pools."""
    import json
    from paper_2201_05587_amd import tune
    tuned_dir = os.path.join(ROOT, "paper_2201_05587_amd", "tuned")
    _, targets, _ = tune.workload("cfg2")
    with open(os.path.join(tuned_dir, "cfg2.json")) as f:
        by_name = {e["name"]: e for e in json.load(f)["kernels"]}
    default_us = [by_name[k.name]["default_us"] for k in targets]
    pools = {n: tune.load_pool(os.path.join(tuned_dir, f"{n}.pool")) for n in ("cfg3", "cfg4", "cfg2", "cfg5")}
    best, scores = tune.choose_donor_pool(targets, default_us, pools)
    # BERT-shaped records share only the classifier's class with a CNN; the conv pools win on their class-E records
    assert scores["cfg3"] == min(scores.values()) and best in ("cfg2", "cfg5") and scores[best] == max(scores.values())
    cost = {}
    for k, us in zip(targets, default_us):
        cost[k.cls] = cost.get(k.cls, 0.0) + us * k.use_count
    total = sum(cost.values())
    for n, pool in pools.items():
        count = {}
        for r in pool:
            count[r.cls] = count.get(r.cls, 0) + 1
        want = S.model_selection_score({c: v / total for c, v in cost.items()}, count)
        assert abs(scores[n] - want) <= 1e-12 * max(1.0, want)


def test_sweep_plan_matches_oracle():
    rng = random.Random(11)
    for it in range(300):
        nk, np_ = rng.randrange(1, 7), rng.randrange(0, 12)
        kc = [rng.randrange(3) for _ in range(nk)]
        pc = [rng.randrange(3) for _ in range(np_)]
        w = [rng.choice([1.0, 2.0, 2.0, 5.5, 9.0]) for _ in range(nk)]
        total = S.evaluation_count(kc, pc) - nk
        budget = rng.choice([0, 1, 2, 3, total - 1, total, total + 3, rng.randrange(0, total + 2)])
        seed = rng.randrange(2 ** 64) if it % 3 else it
        for prio in (0, 1):
            want = S.sweep_plan(kc, w, pc, budget, bool(prio), seed)
            got, selected = api.tt_sweep_plan(kc, w, pc, budget, prio, seed)
            assert got == want, (kc, pc, w, budget, prio, seed)
            assert selected == sum(map(sum, want))
    assert api.tt_sweep_plan([1, 1], None, [1, 1, 1], 2, 0, 5)[1] == 2
    with pytest.raises(api.TTError):
        api.tt_sweep_plan([1], None, [1], 1, 1, 0)   # prioritising needs the weights


def test_selection_with_untried_pairs_matches_oracle():
    rng = random.Random(17)
    for _ in range(100):
        nk, np_ = rng.randrange(1, 5), rng.randrange(1, 7)
        kc = [rng.randrange(2) for _ in range(nk)]
        pc = [rng.randrange(2) for _ in range(np_)]
        pair = [[rng.choice([-1.0, -3.0, 1.0, 2.0, 3.0]) for _ in range(np_)] for _ in range(nk)]
        default = [rng.choice([1.5, 2.5]) for _ in range(nk)]
        want = S.select(kc, pc, pair, default)
        got = api.tt_sweep_select(kc, pc, pair, default)
        assert [tuple(g) for g in got] == [tuple(w) for w in want]


def test_refine_space_matches_oracle():
    rng = random.Random(23)
    checked = 0
    for _ in range(600):
        cls = rng.randrange(S.NUM_CLASSES)
        rec = random_record(rng, cls)
        if not S.record_is_well_formed(rec):
            with pytest.raises(api.TTError):
                api.tt_refine_space(to_c_record(rec))
            continue
        want = S.refine_neighbours(rec)
        got = [r.knobs() for r in api.tt_refine_space(to_c_record(rec))]
        key = lambda r: tuple(r[f] for f in S.RECORD_FIELDS)
        assert sorted(map(key, got)) == sorted(map(key, want)), rec
        assert len(set(map(key, got))) == len(got)
        checked += 1
    assert checked > 200
