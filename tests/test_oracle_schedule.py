"""Pins of the integer oracle (schedule re-application, index map, sweep selection, Eq. 1).

Fixtures under tests/golden/ hold what the paper prints (Section 4.1's Split
example, Algorithm 1's split chains, Table 2 / Table 3, Section 5.2's pair
counts); the rest are invariants checked by brute force.
"""
import itertools
import os

import pytest

from oracle import schedule as S
from paper_2201_05587_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def lines(name):
    with open(os.path.join(GOLD, name)) as f:
        for ln in f:
            ln = ln.strip()
            if ln and not ln.startswith("#"):
                yield ln


def oshape(k: wl.Kernel):
    s = k.shape
    if k.is_conv():
        return S.conv_shape(s.n, s.c, s.h, s.w, s.k, s.r, s.s, s.stride_h, s.stride_w, s.pad_h, s.pad_w, s.dtype)
    return S.gemm_shape(s.batch, s.m, s.n, s.k, s.trans_b, s.dtype)


# ---- Split (Section 4.1 / 4.2) -------------------------------------------------------------------
def test_split_examples_from_the_paper():
    for ln in lines("split_examples.txt"):
        kind, extent, a, b, exp = ln.split()
        if kind == "fixed":
            assert S.split_fixed(int(extent), int(a), int(b)) == bool(int(exp))
        else:
            res = S.split(int(extent), int(a), strict=True)
            assert (-1 if res is None else res[0]) == int(exp)
            if res is not None:
                assert res[1] == int(a) and res[0] * res[1] == int(extent)


def test_split_guarded_tail_reading():
    assert S.split(12, 8, strict=False) == (2, 8)      # ceil(12 / 8) outer iterations, tail guarded
    assert S.split(4, 8, strict=False) is None          # factor larger than the loop: always invalid
    assert S.split(49, 32, strict=False) == (2, 32)     # 7x7 map: 32 fits with a 17-row tail, 64 does not
    assert S.split(49, 64, strict=False) is None


def test_algorithm1_split_chains_transfer_both_ways():
    fused = {}
    outer = {}
    for ln in lines("alg1_split_chains.txt"):
        if ln.startswith("fused"):
            _, name, f512, f1024 = ln.split()
            fused[name] = (int(f512), int(f1024))
            continue
        head, e512, e1024 = [p.strip() for p in ln.split("|")]
        name, axis, start, factors = head.split()
        factors = [int(v) for v in factors.split(",")]
        for size, exp in ((512, e512), (1024, e1024)):
            extent = size if start == "full" else int(start)
            got = S.replay_split_chain(extent, factors, strict=True)
            assert got is not None, (name, axis, size)          # every transformation stays valid
            assert list(got) == [int(v) for v in exp.split(",")], (name, axis, size)
            prod = 1
            for v in got:
                prod *= v
            assert prod == extent
            outer[(name, axis, size)] = got[0]
    for name, (f512, f1024) in fused.items():
        assert outer[(name, "N", 512)] * outer[(name, "M", 512)] == f512
        assert outer[(name, "N", 1024)] * outer[(name, "M", 1024)] == f1024


# ---- apply ---------------------------------------------------------------------------------------
E = S.CLS_CONV2D_BIAS_RELU


def cfg1_shape():
    return S.conv_shape(1, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, S.DT_F32)


def test_apply_derives_outer_extents_from_the_target():
    rec = S.record(E, S.SK_MFMA, 64, 32, 32, 32, 32, 32, 2, 1, 4, 2, 2)
    donor = S.apply(rec, E, S.conv_shape(1, 128, 28, 28, 128, 3, 3, 1, 1, 1, 1))
    target = S.apply(rec, E, cfg1_shape())
    assert donor["status"] == S.OK and target["status"] == S.OK
    # inner factors unchanged, outer extents follow the shape
    for f in ("tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "mfma"):
        assert donor[f] == target[f] == rec[f]
    assert (donor["M"], donor["N"], donor["K"]) == (784, 128, 1152)
    assert (target["M"], target["N"], target["K"]) == (3136, 64, 576)
    assert (donor["tiles_m"], donor["tiles_n"], donor["k_tiles"]) == (13, 4, 36)
    assert (target["tiles_m"], target["tiles_n"], target["k_tiles"]) == (49, 2, 18)
    assert donor["tail_m"] == 784 - 12 * 64 and target["tail_m"] == 64
    assert target["eff_split_k"] == 2 and target["k_iters"] == 9
    assert target["grid"] == 49 * 2 * 2 and target["block"] == 64 * 2
    assert target["workspace_bytes"] == 4 * 2 * 3136 * 64


def test_factor_larger_than_loop_is_invalid_and_wrong_class_is_mismatch():
    s7 = S.conv_shape(1, 512, 7, 7, 512, 3, 3, 1, 1, 1, 1)  # M = 49
    assert S.apply(S.record(E, tile_m=64), E, s7)["status"] == S.ERR_INVALID_SCHEDULE
    assert S.apply(S.record(E, tile_m=64), E, s7)["reason"] == S.R_FACTOR_GT_M
    ok = S.apply(S.record(E, tile_m=32, wave_m=32), E, s7)
    assert ok["status"] == S.OK and ok["tiles_m"] == 2 and ok["tail_m"] == 17
    strict = S.apply(S.record(E, tile_m=32, wave_m=32), E, s7, S.STRICT_DIVISIBLE)
    assert strict["status"] == S.ERR_INVALID_SCHEDULE and strict["reason"] == S.R_NOT_DIVISIBLE
    pw = S.conv_shape(1, 16, 112, 112, 96, 1, 1)  # K = 16
    assert S.apply(S.record(S.CLS_CONV2D_BIAS_RELU6, tile_k=32), S.CLS_CONV2D_BIAS_RELU6, pw)["reason"] == S.R_FACTOR_GT_K
    assert S.apply(S.record(E, tile_n=128, wave_n=32), E, cfg1_shape())["reason"] == S.R_FACTOR_GT_N
    # Section 4.2: a class-E schedule on a dense (class D) kernel is always invalid
    d = S.gemm_shape(1, 64, 1000, 512, 1)
    assert S.apply(S.record(E), S.CLS_DENSE_ADD, d)["status"] == S.ERR_CLASS_MISMATCH
    assert S.apply(S.record(S.CLS_CONV2D_BIAS_ADD_RELU), E, cfg1_shape())["status"] == S.ERR_CLASS_MISMATCH


def test_split_of_the_reduction():
    sh = S.conv_shape(1, 64, 56, 56, 128, 1, 1, 2, 2)  # K = 64
    r = S.record(S.CLS_CONV2D_ADD, tile_k=32, split_k=4)
    p = S.apply(r, S.CLS_CONV2D_ADD, sh)
    assert p["status"] == S.ERR_INVALID_SCHEDULE and p["reason"] == S.R_SPLIT_K  # only 2 K tiles
    p = S.apply(S.record(E, tile_k=32, split_k=4), E, cfg1_shape())   # 18 K tiles
    assert (p["k_iters"], p["eff_split_k"]) == (5, 4)
    p = S.apply(S.record(E, tile_k=32, split_k=7), E, cfg1_shape())   # ceil(18/7)=3 -> 6 non-empty splits
    assert (p["k_iters"], p["eff_split_k"]) == (3, 6)
    # strict reading: the split has to divide the K tiles as well
    assert S.apply(S.record(E, tile_k=32, split_k=4), E, cfg1_shape(), S.STRICT_DIVISIBLE)["reason"] == S.R_NOT_DIVISIBLE
    assert S.apply(S.record(E, tile_k=32, split_k=3), E, cfg1_shape(), S.STRICT_DIVISIBLE)["status"] == S.OK


def test_the_reduction_of_a_convolution_is_c_r_s_whatever_the_channel_count():
    """Factors are compared with the fused extents of Algorithm 2's nest: K = c * r * s, also where a
    pixel's channels do not fill a memory access (3-channel stem, 36 channels in bf16)."""
    stem = S.conv_shape(1, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)
    p = S.apply(S.record(E, tile_k=16), E, stem)
    assert (p["status"], p["M"], p["N"], p["K"]) == (S.OK, 112 * 112, 64, 147)
    assert (p["k_tiles"], p["tail_k"]) == (10, 147 - 9 * 16)
    assert S.apply(S.record(E, tile_k=128), E, stem)["k_tiles"] == 2
    pw = S.conv_shape(1, 36, 14, 14, 576, 1, 1, dtype=S.DT_BF16)
    p = S.apply(S.record(E, tile_k=32), E, pw)
    assert (p["K"], p["k_tiles"], p["tail_k"]) == (36, 2, 4)
    assert S.apply(S.record(E, tile_k=64), E, pw)["reason"] == S.R_FACTOR_GT_K
    assert S.apply(S.record(E), E, cfg1_shape())["K"] == 64 * 3 * 3


def test_depthwise_vector_width_is_reformulated_to_the_channel_count():
    """Section 4.1: a knob is reformulated where it can be; the vector width of the depthwise sketch
    becomes the widest power of two that divides the channel count, and the workgroup's lanes then
    cover tile_k times as many planes."""
    dw = S.CLS_DWCONV_BIAS_RELU6
    def plan(c, vec, tile_k=16, n=2):
        rec = S.record(dw, S.SK_DWCONV, 4, 4, tile_k, 1, 1, 0, 1, 0, vec, 1, 1)
        return S.apply(rec, dw, S.conv_shape(n, c, 14, 14, c, 3, 3, 1, 1, 1, 1))
    assert plan(96, 4)["tile_k"] == 64 and plan(96, 2)["tile_k"] == 32 and plan(96, 1)["tile_k"] == 16
    assert plan(36, 8)["tile_k"] == 64       # fp32: at most four elements per access
    assert plan(18, 4)["tile_k"] == 32 and plan(27, 4)["tile_k"] == 16
    p = plan(96, 4)
    assert (p["K"], p["k_tiles"], p["block"], p["grid"]) == (192, 3, 16 * 16, 4 * 4 * 3)
    assert plan(8, 4, tile_k=16, n=1)["reason"] == S.R_FACTOR_GT_K   # 64 planes asked of 8


def test_malformed_records_and_shapes_are_argument_errors():
    assert S.apply(S.record(E, wave_m=48), E, cfg1_shape())["status"] == S.ERR_BAD_ARG
    assert S.apply(S.record(E, mfma=8), E, cfg1_shape())["status"] == S.ERR_BAD_ARG
    assert S.apply(S.record(E, tile_m=256, tile_n=256, wave_m=16, wave_n=16), E, cfg1_shape())["status"] == S.ERR_BAD_ARG
    assert S.apply(S.record(E, vec=3), E, cfg1_shape())["status"] == S.ERR_BAD_ARG
    assert S.apply(S.record(E), E, S.conv_shape(1, 0, 8, 8, 4, 3, 3))["status"] == S.ERR_BAD_ARG
    assert S.apply(S.record(E), E, S.conv_shape(1, 4, 2, 2, 4, 5, 5))["status"] == S.ERR_BAD_ARG
    assert S.apply(S.record(E), 99, cfg1_shape())["status"] == S.ERR_BAD_ARG


def all_cfg_kernels():
    ks = [wl.cfg1_target(), wl.cfg1_donor()] + wl.resnet18_kernels() + wl.resnet50_kernels()
    ks += wl.bert_kernels() + wl.bert_kernels(seq=256) + wl.mobilenetv2_kernels(1) + wl.mobilenetv2_kernels(16)
    ks += wl.resnet50_kernels(32, wl.BF16, with_dense=False)
    for i in range(3):
        ks += wl.synthetic_network(i)
    return ks


def test_default_schedule_is_valid_for_every_configured_shape():
    for k in all_cfg_kernels():
        rec = S.default_schedule(k.cls, oshape(k))
        p = S.apply(rec, k.cls, oshape(k))
        assert p["status"] == S.OK, (k.name, rec, p)
        assert S.apply(rec, k.cls, oshape(k), S.STRICT_DIVISIBLE)["status"] in (S.OK, S.ERR_INVALID_SCHEDULE)
    # and for degenerate tiny shapes, through the one-thread-per-output record
    tiny = S.conv_shape(1, 2, 4, 4, 3, 3, 3, 1, 1, 1, 1)
    assert S.default_schedule(E, tiny)["sketch"] == S.SK_DIRECT
    assert S.apply(S.default_schedule(E, tiny), E, tiny)["status"] == S.OK
    assert S.apply(S.default_schedule(S.CLS_DENSE_ADD, S.gemm_shape(1, 1, 3, 5, 1)), S.CLS_DENSE_ADD,
                   S.gemm_shape(1, 1, 3, 5, 1))["status"] == S.OK


# ---- index map -----------------------------------------------------------------------------------
def check_cover(plan):
    """Every (batch, m, n, k) cell is owned by exactly one workgroup; the map is a bijection."""
    seen_tiles = set()
    area = 0
    for wg in range(plan["grid"]):
        b, z, m0, me, n0, ne, k0, ke = S.plan_tile(plan, wg)
        assert me >= 1 and ne >= 1 and ke >= 1
        assert m0 + me <= plan["M"] and n0 + ne <= plan["N"] and k0 + ke <= plan["K"]
        assert m0 % plan["tile_m"] == 0 and n0 % plan["tile_n"] == 0
        key = (b, z, m0, n0, k0)
        assert key not in seen_tiles
        seen_tiles.add(key)
        area += me * ne * ke
    slabs_hi = plan["batch"] if plan["sketch"] != S.SK_DWCONV else 1
    assert area == slabs_hi * plan["M"] * plan["N"] * plan["K"]


@pytest.mark.parametrize("order", range(6))
def test_index_map_is_a_bijection_that_tiles_the_iteration_space(order):
    shapes = [
        (E, S.conv_shape(1, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1)),
        (E, S.conv_shape(1, 512, 7, 7, 512, 3, 3, 1, 1, 1, 1)),
        (E, S.conv_shape(1, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)),
        (S.CLS_BATCH_MATMUL, S.gemm_shape(5, 128, 64, 128, 0, S.DT_BF16)),
        (S.CLS_DENSE_ADD, S.gemm_shape(1, 1024, 1000, 768, 1, S.DT_BF16)),
    ]
    for (cls, sh), (tm, tn, sk) in itertools.product(shapes, [(32, 32, 1), (32, 64, 3), (16, 16, 2)]):
        rec = S.record(cls, S.SK_MFMA, tm, tn, 32, 16, 16, 16, sk, order, 4, 1, 2)
        p = S.apply(rec, cls, sh)
        if p["status"] != S.OK:
            continue
        check_cover(p)
    dw = S.conv_shape(2, 48, 14, 14, 48, 3, 3, 2, 2, 1, 1)
    p = S.apply(S.record(S.CLS_DWCONV_BIAS_RELU6, S.SK_DWCONV, 4, 4, 8, 1, 1, 0, 1, order, 1, 1, 1),
                S.CLS_DWCONV_BIAS_RELU6, dw)
    assert p["status"] == S.OK
    check_cover(p)


def test_index_map_orders_by_hand():
    sh = S.gemm_shape(1, 96, 64, 64, 1)   # 3 x 2 tiles of 32
    def tiles(order):
        p = S.apply(S.record(S.CLS_DENSE_ADD, S.SK_MFMA, 32, 32, 16, 32, 32, 16, 1, order), S.CLS_DENSE_ADD, sh)
        return [(t[2] // 32, t[4] // 32) for t in (S.plan_tile(p, w) for w in range(p["grid"]))]
    assert tiles(0) == [(0, 0), (1, 0), (2, 0), (0, 1), (1, 1), (2, 1)]
    assert tiles(1) == [(0, 0), (0, 1), (1, 0), (1, 1), (2, 0), (2, 1)]
    assert tiles(2) == tiles(0)  # fewer than GROUP_M tiles: one band
    # 6 workgroups over 8 XCDs: XCD x holds logical id x
    assert tiles(3) == tiles(0)
    sh = S.gemm_shape(1, 32 * 20, 32, 64, 1)  # 20 x 1 tiles -> XCD x gets ids {x, x+8, x+16}
    p = S.apply(S.record(S.CLS_DENSE_ADD, S.SK_MFMA, 32, 32, 16, 32, 32, 16, 1, 3), S.CLS_DENSE_ADD, sh)
    got = [S.plan_tile(p, w)[2] // 32 for w in range(20)]
    # XCDs 0..3 own 3 tiles, 4..7 own 2: XCD0 -> 0,1,2; XCD1 -> 3,4,5; ...; XCD4 -> 12,13; ...
    assert got[0] == 0 and got[8] == 1 and got[16] == 2 and got[1] == 3 and got[4] == 12 and got[12] == 13
    assert sorted(got) == list(range(20))


def test_grouped_order_walks_bands_of_eight():
    sh = S.gemm_shape(1, 32 * 10, 32 * 3, 64, 1)
    p = S.apply(S.record(S.CLS_DENSE_ADD, S.SK_MFMA, 32, 32, 16, 32, 32, 16, 1, 2), S.CLS_DENSE_ADD, sh)
    got = [(t[2] // 32, t[4] // 32) for t in (S.plan_tile(p, w) for w in range(p["grid"]))]
    assert got[:9] == [(0, 0), (1, 0), (2, 0), (3, 0), (4, 0), (5, 0), (6, 0), (7, 0), (0, 1)]
    assert got[24:] == [(8, 0), (9, 0), (8, 1), (9, 1), (8, 2), (9, 2)]


# ---- sweep selection (Section 4.3) ---------------------------------------------------------------
def test_selection_on_a_hand_made_time_matrix():
    kc = [1, 1, 2, 4]
    pc = [1, 1, 0, 4, 1]
    pair = [
        [5.0, 3.0, 9.0, 9.0, -1.0],   # donor 1 wins; donor 4 invalid; donors 2, 3 are other classes
        [7.0, 7.5, 0.1, 0.1, 8.0],    # default (6.0) wins; cheap times of other classes are ignored
        [1.0, 1.0, 1.0, 1.0, 1.0],    # class 2 has no donor -> default
        [9.0, 9.0, 9.0, 2.0, 9.0],    # tie with the default -> default
    ]
    default = [4.0, 6.0, 3.0, 2.0]
    rows = S.select(kc, pc, pair, default)
    assert rows == [(1, 3.0, 2, 1), (-1, 6.0, 3, 0), (-1, 3.0, 0, 0), (-1, 2.0, 1, 0)]
    pair[0][0] = 3.0  # equal donors: lowest index
    assert S.select(kc, pc, pair, default)[0][0] == 0
    assert S.select(kc, pc, pair, default, allow_slower_than_default=True)[1] == (0, 7.0, 3, 0)


def test_selection_leaves_untried_pairs_out_of_both_counts():
    kc, pc = [1, 1], [1, 1, 1]
    pair = [[5.0, S.NOT_TRIED, -1.0], [S.NOT_TRIED, S.NOT_TRIED, S.NOT_TRIED]]
    assert S.select(kc, pc, pair, [6.0, 2.0]) == [(0, 5.0, 1, 1), (-1, 2.0, 0, 0)]


# ---- cheaper sweeps (Sections 5.5, 4.4.2) and refinement (Section 6) ------------------------------
def test_splitmix64_reference_values():
    """First outputs of SplitMix64 from state 0 (the values every published implementation prints) and from
    the state 1234567: the generator advances its state by the golden-ratio constant before each output,
    so output number n of seed s is splitmix64(s + (n - 1) * gamma)."""
    gamma = 0x9E3779B97F4A7C15
    want0 = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [S.splitmix64((n * gamma) & S.MASK64) for n in range(3)] == want0
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423]
    assert [S.splitmix64((1234567 + n * gamma) & S.MASK64) for n in range(3)] == want


def test_sweep_plan_budget_and_priority_rules():
    kc = [1, 1, 2, 4]
    pc = [1, 1, 0, 4, 1, 2, 1]
    weights = [10.0, 30.0, 30.0, 5.0]
    same = [(k, p) for k in range(4) for p in range(7) if pc[p] == kc[k]]
    assert len(same) == 4 + 4 + 1 + 1
    def picked(mask):
        return [(k, p) for k in range(4) for p in range(7) if mask[k][p]]
    # no budget, or one that covers everything: every same-class pair and nothing else
    for budget in (0, -1, 10, 99):
        assert picked(S.sweep_plan(kc, weights, pc, budget, False, 7)) == same
    # a budget keeps exactly that many same-class pairs: the ones with the smallest keys
    for budget in range(1, 10):
        got = picked(S.sweep_plan(kc, weights, pc, budget, False, 7))
        assert len(got) == budget and set(got) <= set(same)
        keys = sorted((S.splitmix64(7 + k * 7 + p + 1), k * 7 + p) for k, p in same)
        assert sorted(k * 7 + p for k, p in got) == sorted(i for _, i in keys[:budget])
        # nested: a larger budget only adds pairs
        assert set(got) <= set(picked(S.sweep_plan(kc, weights, pc, budget + 1, False, 7)))
    assert picked(S.sweep_plan(kc, weights, pc, 5, False, 7)) != picked(S.sweep_plan(kc, weights, pc, 5, False, 8))
    # priority: kernel 1 (weight 30, lower index than kernel 2) is served first, then 2, then 0, then 3
    got = picked(S.sweep_plan(kc, weights, pc, 4, True, 7))
    assert got == [(1, 0), (1, 1), (1, 4), (1, 6)]
    got = picked(S.sweep_plan(kc, weights, pc, 5, True, 7))
    assert got == [(1, 0), (1, 1), (1, 4), (1, 6), (2, 5)]
    got = picked(S.sweep_plan(kc, weights, pc, 7, True, 7))
    assert [q for q in got if q[0] != 0] == [(1, 0), (1, 1), (1, 4), (1, 6), (2, 5)] and len(got) == 7
    assert sum(1 for q in got if q[0] == 0) == 2 and all(q[0] != 3 for q in got)


def test_uniform_sampling_is_close_to_uniform():
    """Each of 200 same-class pairs is kept about budget/total of the time over 400 seeds (a biased key, an
    index reused as a key or a sort on the wrong field would fail this)."""
    kc, pc = [0] * 10, [0] * 20
    hits = [0] * 200
    for seed in range(400):
        m = S.sweep_plan(kc, None, pc, 50, False, seed * 1000)
        for k in range(10):
            for p in range(20):
                hits[k * 20 + p] += m[k][p]
    assert sum(hits) == 400 * 50
    assert min(hits) > 60 and max(hits) < 145   # mean 100, sd 8.7: six sigma


def test_refinement_neighbourhood_by_hand():
    base = S.record(E, S.SK_MFMA, 64, 64, 32, 32, 32, 16, 2, 1, 4, 8, 2)
    near = S.refine_neighbours(base)
    def has(**ch):
        return dict(base, **ch) in near
    assert all(S.record_is_well_formed(r) for r in near) and base not in near
    assert all(sum(1 for f in S.RECORD_FIELDS if r[f] != base[f]) == 1 for r in near)
    assert has(tile_m=128) and has(tile_m=32) and has(tile_n=128) and has(tile_k=64) and has(tile_k=16)
    assert has(wave_m=64) and has(wave_m=16) and has(wave_n=16)
    assert has(mfma=32) and has(split_k=1) and has(split_k=3) and not has(split_k=4)
    assert all(has(order=o) for o in (0, 2, 3, 4, 5)) and has(stages=1) and has(stages=3) and has(unroll=1)
    assert has(vec=8) and has(vec=2)
    # 5 orders + 2 stages + unroll + mfma + 2 splits + 2 vec + tile_m 2 + tile_n 2 + tile_k 2 + wave_m 2 + wave_n 2
    assert len(near) == 5 + 2 + 1 + 1 + 2 + 2 + 2 + 2 + 2 + 2 + 2
    # at the edges of the record format steps fall away: 16-wide tiles cannot shrink, a 32-block cannot halve its wave
    small = S.record(E, S.SK_MFMA, 32, 32, 16, 32, 32, 32, 1, 0, 1, 1, 1)
    near = S.refine_neighbours(small)
    assert dict(small, wave_m=16) not in near and dict(small, tile_k=8) not in near and dict(small, stages=0) not in near
    assert dict(small, split_k=2) in near and dict(small, vec=2) in near and dict(small, unroll=8) in near
    assert S.refine_neighbours(S.record(E, S.SK_DIRECT, 1, 1, 1, 1, 1, 0, 1, 0, 1, 1, 1)) == []


def parse_table2():
    models, pairs, kernels, r18 = {}, [], {}, {}
    for ln in lines("table2_model_classes.txt"):
        tok = ln.split()
        if tok[0] == "pairs":
            pairs.append((tok[1], tok[2], int(tok[3]), int(tok[4])))
        elif tok[0] == "kernels":
            kernels[tok[1]] = int(tok[2])
        elif tok[0] == "resnet18":
            r18 = {t.split(":")[0]: int(t.split(":")[1]) for t in tok[1:]}
        else:
            left, tuning, top3 = [p.strip() for p in ln.split("|")]
            lt = left.split()
            cls = {t.split(":")[0]: (int(t.split(":")[1]), int(t.split(":")[2])) for t in lt[2:]}
            models[lt[0]] = dict(name=lt[1], cls=cls, tuning=tuning, top3=top3.split())
    return models, pairs, kernels, r18


def test_evaluation_counts_match_the_papers_pair_counts():
    models, pairs, kernels, r18 = parse_table2()

    def kernel_list(m):
        return [c for c, (n, _) in models[m]["cls"].items() for _ in range(n)]
    for target, donor, n_pairs, n_kernels in pairs:
        assert len(kernel_list(target)) == n_kernels
        assert S.evaluation_count(kernel_list(target), kernel_list(donor)) == n_pairs
    assert len(kernel_list("M7")) == kernels["M7"]
    # ResNet18 with ResNet50's schedules (Section 4.3): A has 4 donors, E 16, B/C/D one each, F none
    r18_list = [c for c, n in r18.items() for _ in range(n)]
    assert len(r18_list) == 18
    assert S.evaluation_count(r18_list, kernel_list("M1")) == 3 * 5 + 8 * 17 + 4 * 1 + 3 * 2


def test_equation1_reproduces_table2_and_table3():
    models, _, _, _ = parse_table2()
    for mid, m in models.items():
        cost = {c: pct / 100.0 for c, (_, pct) in m["cls"].items()}
        scores = {}
        for tid, t in models.items():
            if tid == mid:
                continue
            scores[tid] = S.model_selection_score(cost, {c: n for c, (n, _) in t["cls"].items()})
        ranked = sorted(scores, key=lambda t: -scores[t])
        assert ranked[0] == m["tuning"], (mid, ranked[:3])
        for pos, want in enumerate(m["top3"]):
            if want != "-":
                assert ranked[pos] == want, (mid, pos, ranked[:3])
