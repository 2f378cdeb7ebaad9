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


def plan_equal(cplan: api.tt_plan, oplan: dict):
    got = cplan.spec()
    assert set(got) == set(S.PLAN_FIELDS)
    diff = {k: (got[k], oplan[k]) for k in S.PLAN_FIELDS if got[k] != oplan[k]}
    assert not diff, diff


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
                    rng.choice([1, 2, 4, 8]), rng.choice([1, 2, 4, 512]), rng.choice([1, 2, 3, 4]))


def test_apply_matches_oracle_bit_for_bit_on_random_records():
    rng = random.Random(20220105)
    kernels = all_cfg_kernels()
    statuses = {}
    for it in range(6000):
        k = rng.choice(kernels)
        rec = random_record(rng, k.cls if rng.random() < 0.9 else rng.randrange(S.NUM_CLASSES))
        flags = S.STRICT_DIVISIBLE if rng.random() < 0.2 else 0
        oplan = S.apply(rec, k.cls, oshape(k), flags)
        cplan = api.tt_schedule_apply(to_c_record(rec), k.cls, k.shape, flags)
        plan_equal(cplan, oplan)
        statuses[oplan["status"]] = statuses.get(oplan["status"], 0) + 1
        if oplan["status"] == S.OK and oplan["sketch"] != S.SK_DIRECT and oplan["grid"] <= 4096 and it % 10 == 0:
            for wg in range(oplan["grid"]):
                assert api.tt_plan_tile(cplan, wg) == S.plan_tile(oplan, wg)
    # the draw must exercise every outcome
    assert all(statuses.get(s, 0) > 50 for s in (S.OK, S.ERR_INVALID_SCHEDULE, S.ERR_CLASS_MISMATCH, S.ERR_BAD_ARG))


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
        plan_equal(cplan, oplan)
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
    # every default matrix-core record of the configured shapes has a compiled variant
    for k in all_cfg_kernels():
        rec = api.tt_schedule_default(k.cls, k.shape)
        plan = api.tt_schedule_apply(rec, k.cls, k.shape)
        assert plan.status == api.TT_OK
        if plan.sketch == api.TT_SK_MFMA:
            assert plan.variant_id >= 0, (k.name, rec)


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
